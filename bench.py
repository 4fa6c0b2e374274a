#!/usr/bin/env python3
"""Benchmark: one MoE layer forward (route -> permute -> gate+up -> down -> combine) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config mixtral] [--T 512]
    python bench.py --grid "mixtral:1,16,64,256,512,4096:0;qwen2moe:512,4096:0,1,1.5,2" [--steps K]

Prints ONE JSON line (or, with --grid, one table row per (shape, T, skew) cell, all cells of a
shape sharing one set of generated weights: that is how the sweeps under profiles/ are made).  `value` is tokens/s of the whole layer with all inputs resident in HBM.
`roofline` is for the dominant kernel (the fused gate+up grouped GEMM), timed inside the timed
region with HIP events recorded by the library on the launch stream.  `cpu_baseline` is the
fp64 numpy oracle timed on this machine's host cores on a bounded token sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import moe_inputs as mi  # noqa: E402

HBM_PEAK_GBS = 8000.0        # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X published dense bf16 MFMA peak


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="mixtral", choices=sorted(mi.PRESETS))
    ap.add_argument("--T", type=int, default=512)
    ap.add_argument("--shape", default="", help="d,F,E,k of a synthetic layer (softmax gating) instead of --config, "
                                                "e.g. the expert-scaling ladder of the paper's Table 5")
    ap.add_argument("--skew", type=float, default=0.0)
    ap.add_argument("--tile-m", type=int, default=0)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=0, help="tokens the oracle's FFN is timed on (0 = auto)")
    ap.add_argument("--row-major", action="store_true",
                    help="feed the GEMMs the row-major [E,N,K] weights instead of the one-time packed copy")
    ap.add_argument("--fuse-combine", action="store_true",
                    help="set MOE_FLAG_FUSE_COMBINE: the weighted combine runs inside the down projection")
    ap.add_argument("--grid", default="",
                    help="sweep instead of one point: 'shape:T,T,...:skew,skew,...;shape:...' with shape a preset or "
                         "d,F,E,k written as custom_d_F_E_k; prints a table, one row per cell")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (torch) so that a rocprofv3 --pmc run of this "
                         "command holds a kernel of known HBM traffic to scale FETCH_SIZE / WRITE_SIZE by")
    return ap.parse_args()


def cpu_baseline(shape, x_cpu, wr_cpu, bias_cpu, seed, sample):
    """The oracle as it stands: routing + permutation on all T tokens, FFN on `sample` tokens."""
    from oracle import moe_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    rng = np.random.default_rng(seed + 17)
    tokens = sorted(rng.choice(shape.T, size=min(sample, shape.T), replace=False).tolist())
    prov = lambda e: tuple(mi.bits(t) for t in mi.make_expert(shape, e, seed))
    t0 = time.perf_counter()
    out = orc.moe_forward(mi.bits(x_cpu), mi.bits(wr_cpu), None if bias_cpu is None else bias_cpu.numpy(), prov,
                          shape.k, shape.gating, tokens=tokens)
    dt = time.perf_counter() - t0
    return {"value": len(tokens) / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"fp64 numpy oracle: routing+permutation of all {shape.T} tokens, expert FFN+combine of "
                      f"{len(tokens)} seeded tokens ({dt:.1f} s, includes regenerating and decoding the experts hit)"}, out


def grid(args):
    """Per-stage timings over a grid of cells in one process (the weights of a shape are generated once)."""
    import paper_2605_23911_amd as moe
    dev = "cuda:0"
    stream = torch.cuda.current_stream()
    flags = moe.FLAG_FUSE_COMBINE if args.fuse_combine else 0

    def ev():
        e = torch.cuda.Event(enable_timing=True)
        e.record(stream)
        return e

    print(f"{'shape':22s} {'T':>5s} {'skew':>4s} {'act':>4s} {'ms/fwd':>8s} {'tokens/s':>10s} | {'route':>6s} {'perm':>6s} "
          f"{'gate_up':>8s} {'down':>8s} {'comb':>6s} (us) | gate+up: vs HBM, vs MFMA | down: vs HBM, vs MFMA | "
          f"layer: vs HBM, vs MFMA", flush=True)
    for part in args.grid.split(";"):
        name, Ts, skews = part.split(":")
        if name.startswith("custom_"):
            d_, F_, E_, k_ = (int(v) for v in name.split("_")[1:])
            base = mi.MoEShape(name, 512, d_, F_, E_, k_)
        else:
            base = mi.PRESETS[name]
        wg = torch.empty((base.E, base.F, base.d), dtype=torch.bfloat16, device=dev)
        wu = torch.empty_like(wg)
        wd = torch.empty((base.E, base.d, base.F), dtype=torch.bfloat16, device=dev)
        mi.make_all_experts(base, args.seed, out=(wg, wu, wd))
        cfg0 = moe.MoEConfig.of(1, base.d, base.F, base.E, base.k, base.gating)
        pk = None
        if not args.row_major:
            pk = torch.empty(moe.packed_weights_size(cfg0), dtype=torch.uint8, device=dev)
            moe.moe_pack_weights(cfg0, wg, wu, wd, pk)
            torch.cuda.synchronize()
            wg = wu = wd = None
        for T in (int(v) for v in Ts.split(",")):
            s = base.with_T(T)
            x, wr = mi.make_x(s, args.seed).to(dev), mi.make_router(s, args.seed).to(dev)
            for skew in (float(v) for v in skews.split(",")):
                b = mi.skew_bias(s, skew, args.seed)
                bias = None if b is None else b.to(dev)
                cfg = moe.MoEConfig.of(s.T, s.d, s.F, s.E, s.k, s.gating, args.tile_m, flags)
                lay = moe.forward_workspace_layout(cfg)
                ws = torch.zeros(lay.total, dtype=torch.uint8, device=dev)
                y = torch.empty((s.T, s.d), dtype=torch.bfloat16, device=dev)
                for _ in range(args.warmup):
                    moe.moe_forward(cfg, x, wr, bias, wg, wu, wd, y, ws, W_packed=pk)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(args.steps):
                    moe.moe_forward(cfg, x, wr, bias, wg, wu, wd, y, ws, W_packed=pk)
                torch.cuda.synchronize()
                ms = (time.perf_counter() - t0) * 1e3 / args.steps
                evs = [[ev() for _ in range(6)] for _ in range(args.steps)]
                torch.cuda.synchronize()
                for row in evs:
                    moe.moe_forward_staged(cfg, x, wr, bias, wg, wu, wd, y, ws, [e.cuda_event for e in row], W_packed=pk)
                torch.cuda.synchronize()
                st = [float(np.median([row[i].elapsed_time(row[i + 1]) for row in evs])) * 1e3 for i in range(5)]
                counts = ws[lay.counts: lay.counts + 4 * s.E].view(torch.int32).cpu().numpy()
                ea, R = int((counts > 0).sum()), s.R
                gub, guf = 4 * s.d * s.F * ea + 2 * R * s.d + 2 * R * s.F, 4 * R * s.d * s.F
                dnb, dnf = 2 * s.d * s.F * ea + 2 * R * s.d + 2 * R * s.F, 2 * R * s.d * s.F
                lb = (6 * s.d * s.F * ea + 2 * s.E * s.d + 2 * s.T * s.d + 2 * R * s.d + 4 * R * s.F + 4 * R * s.d
                      + 2 * s.T * s.d + 16 * R)
                lf = s.T * (6 * s.k * s.d * s.F + 2 * s.E * s.d)
                hb = lambda nbytes, us: nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS
                mf = lambda flops, us: flops / (us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS
                print(f"{name:22s} {T:5d} {skew:4.1f} {ea:4d} {ms:8.4f} {s.T / (ms * 1e-3):10.0f} | {st[0]:6.1f} {st[1]:6.1f} "
                      f"{st[2]:8.1f} {st[3]:8.1f} {st[4]:6.1f}      |     {hb(gub, st[2]):.3f}  {mf(guf, st[2]):.3f}      |   "
                      f"{hb(dnb, st[3]):.3f}  {mf(dnf, st[3]):.3f}    |    {hb(lb, ms * 1e3):.3f}  {mf(lf, ms * 1e3):.3f}", flush=True)
                del ws, y
        del pk, wg, wu, wd
        torch.cuda.empty_cache()


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no expert sharding, no collectives); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    import paper_2605_23911_amd as moe
    moe.lib()   # raises if the HIP library has not been built: there is no fallback

    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.grid:
        return grid(args)
    if args.shape:
        d_, F_, E_, k_ = (int(v) for v in args.shape.split(","))
        s = mi.MoEShape(f"d{d_}-F{F_}-E{E_}-k{k_}", args.T, d_, F_, E_, k_)
    else:
        s = mi.PRESETS[args.config].with_T(args.T)
    x_cpu, wr_cpu = mi.make_x(s, args.seed), mi.make_router(s, args.seed)
    bias_cpu = mi.skew_bias(s, args.skew, args.seed)
    x, wr = x_cpu.to(dev), wr_cpu.to(dev)
    bias = None if bias_cpu is None else bias_cpu.to(dev)
    wg = torch.empty((s.E, s.F, s.d), dtype=torch.bfloat16, device=dev)
    wu = torch.empty((s.E, s.F, s.d), dtype=torch.bfloat16, device=dev)
    wd = torch.empty((s.E, s.d, s.F), dtype=torch.bfloat16, device=dev)
    mi.make_all_experts(s, args.seed, out=(wg, wu, wd))
    cfg = moe.MoEConfig.of(s.T, s.d, s.F, s.E, s.k, s.gating, args.tile_m,
                           moe.FLAG_FUSE_COMBINE if args.fuse_combine else 0)
    packed = None
    if not args.row_major:      # model-load-time step, outside every timed region: same values, re-ordered
        packed = torch.empty(moe.packed_weights_size(cfg), dtype=torch.uint8, device=dev)
        moe.moe_pack_weights(cfg, wg, wu, wd, packed)
        torch.cuda.synchronize()
        wg = wu = wd = None
    lay = moe.forward_workspace_layout(cfg)
    ws = torch.zeros(lay.total, dtype=torch.uint8, device=dev)
    y = torch.empty((s.T, s.d), dtype=torch.bfloat16, device=dev)
    stream = torch.cuda.current_stream()

    def new_event():
        ev = torch.cuda.Event(enable_timing=True)
        ev.record(stream)          # creates the underlying hipEvent_t; the library re-records it
        return ev

    for _ in range(args.warmup):
        moe.moe_forward(cfg, x, wr, bias, wg, wu, wd, y, ws, W_packed=packed)
    torch.cuda.synchronize()

    # ---- timed region: K steps; events [2] and [3] bracket the gate+up kernel of every step
    K = args.steps
    ev_a = [new_event() for _ in range(K)]
    ev_b = [new_event() for _ in range(K)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        moe.moe_forward_staged(cfg, x, wr, bias, wg, wu, wd, y, ws,
                               [None, None, ev_a[i].cuda_event, ev_b[i].cuda_event, None, None], W_packed=packed)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / K
    gate_up_ms = float(np.mean([a.elapsed_time(b) for a, b in zip(ev_a, ev_b)]))

    if args.calibrate_copy:
        src = torch.ones(1 << 29, dtype=torch.bfloat16, device=dev)     # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.neg(src, out=dst)        # one elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    # ---- per-stage breakdown (outside the timed region)
    evs = [[new_event() for _ in range(6)] for _ in range(10)]
    torch.cuda.synchronize()
    for row in evs:
        moe.moe_forward_staged(cfg, x, wr, bias, wg, wu, wd, y, ws, [e.cuda_event for e in row], W_packed=packed)
    torch.cuda.synchronize()
    names = ["route", "permute", "gate_up", "down", "combine"]
    stages = {n: float(np.median([row[i].elapsed_time(row[i + 1]) for row in evs])) for i, n in enumerate(names)}
    stages["total_events"] = float(np.median([row[0].elapsed_time(row[5]) for row in evs]))

    # ---- algorithmic work from the actual routing
    counts = ws[lay.counts: lay.counts + 4 * s.E].view(torch.int32).cpu().numpy()
    e_active = int((counts > 0).sum())
    R = s.R
    gate_up_bytes = 4 * s.d * s.F * e_active + 2 * R * s.d + 2 * R * s.F       # weights once, token rows in, h out
    gate_up_flops = 4 * R * s.d * s.F
    # weights once, router weights, x (router), R gathered token rows (gate+up), h and y_perm written + read,
    # y, index/weight arrays.  No permuted copy of x is written (the gather is folded into gate+up).
    layer_bytes = (6 * s.d * s.F * e_active + 2 * s.E * s.d + 2 * s.T * s.d + 2 * R * s.d + 2 * 2 * R * s.F
                   + 2 * 2 * R * s.d + 2 * s.T * s.d + 16 * R)
    layer_flops = s.T * (6 * s.k * s.d * s.F + 2 * s.E * s.d)
    mean_rows = R / max(e_active, 1)
    if mean_rows > 312:      # ridge point 2.5 PFLOP/s / 8 TB/s
        ach = gate_up_flops / (gate_up_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": ach / MFMA_BF16_PEAK_TFLOPS, "traffic": None}
    else:
        ach = gate_up_bytes / (gate_up_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": ach / HBM_PEAK_GBS, "traffic": None}
    kname = moe.ffn_kernel_name(cfg, 0, packed is not None)
    # HBM bytes per launch from rocprofv3 --pmc counters: they cannot be read from inside this process, so the figure
    # of the committed counter run (profiles/mixtral_T512_hbm_traffic.txt) is reported, and only for the workload and
    # the kernel instance it was taken on: any other point, or a renamed kernel, reports null rather than a stale number.
    try:
        rec = json.load(open(os.path.join(ROOT, "profiles", "traffic.json"))).get(
            f"{s.name} T={s.T} {'packed' if packed is not None else 'row-major'}")
        if rec and rec["kernel"] == kname and args.skew == 0.0 and args.tile_m == 0 and not args.fuse_combine:
            roofline["traffic"] = rec["traffic_bytes"]
            roofline["traffic_source"] = rec.get("source", "profiles/traffic.json")
    except (OSError, ValueError, KeyError):
        pass
    roofline.update({"kernel": kname, "kernel_ms": gate_up_ms,
                     "algorithmic_bytes": gate_up_bytes, "algorithmic_flops": gate_up_flops,
                     "active_experts": e_active})

    result = {
        "metric": "moe_layer_forward_tokens_per_s", "value": s.T / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{s.name}-shaped MoE layer forward, T={s.T} tokens, d={s.d}, F={s.F}, E={s.E}, "
                               f"top-k={s.k}, gating={s.gating}, skew={args.skew}, seed={args.seed}",
                   "tile_m": moe.tile_m(cfg), "weights": "row-major" if args.row_major else "packed once at load"},
        "roofline": roofline,
        "layer": {"hbm_frac": layer_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                  "mfma_frac": layer_flops / (ms_per_step * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                  "algorithmic_bytes": layer_bytes, "algorithmic_flops": layer_flops},
        "stages_ms": stages,
    }
    if not args.no_cpu_baseline:
        sample = args.cpu_sample or min(s.T, 1024)
        result["cpu_baseline"], ref = cpu_baseline(s, x_cpu, wr_cpu, bias_cpu, args.seed, sample)
        yb = y.cpu().view(torch.int16).numpy().view(np.uint16)[ref["tokens"]]
        yg = (yb.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
        result["parity_max_rel_err_sampled"] = float(np.abs(yg - ref["y"]).max() / np.abs(ref["y"]).max())
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
