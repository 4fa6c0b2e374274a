"""GPU parity: every stage of the HIP path, and the whole layer, against the fp64 CPU oracle on
the same seeded bf16 inputs.  Integer results (expert indices, counts, offsets, permutation,
block schedule, gathered rows) must be bit-exact; float results within the stated tolerances:
    topk_w : |gpu - ref| <= 1e-6            (fp64 gate arithmetic, one rounding to fp32)
    h, y_perm, y : max|gpu - ref| <= 1e-2 * max|ref|   (the benchmark contract's bound; the
        arithmetic gives ~2^-9 per bf16 rounding of h, y_perm and y plus fp32 accumulation)
"""
import os
import sys

import numpy as np
import pytest
import torch

sys.path.insert(0, os.path.dirname(__file__))

import moe_inputs as mi
from oracle import moe_oracle as orc

pytestmark = pytest.mark.gpu

REL = 1e-2
GAP_MIN = 1e-9   # top-(k+1) logit gaps far above fp64 summation noise certify the index parity


@pytest.fixture(scope="module")
def G():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2605_23911_amd as moe
    moe.lib()   # fail loudly here if the HIP library is missing
    import gpu_util
    return gpu_util


def _say(msg):
    print(f"[gpu-parity] {msg}", flush=True)


def _relmax(got, ref):
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))


def _oracle_full(layer, **kw):
    s = layer.shape
    return orc.moe_forward(layer.x_bits, layer.wr_bits, layer.bias_np, layer.expert_bits, s.k, s.gating,
                           keep_h=True, **kw)


def _check_routing(out, ref, layer):
    assert ref["min_gap"].min() > GAP_MIN, "seeded logits too close to certify index parity"
    assert np.array_equal(out["topk_idx"], ref["topk_idx"])
    assert np.abs(out["topk_w"].astype(np.float64) - ref["topk_w"]).max() <= 1e-6
    for name in ("counts", "offsets", "row_of", "src_of"):
        assert np.array_equal(out[name], ref[name]), name
    # moe_forward folds the row gather into the gate+up loads and writes no x_perm; the copy that
    # moe_permute makes is checked where that entry point is tested.


def _check_floats(out, ref, layer, G, tokens=None):
    """h and y_perm rows of the checked tokens, and y, against the oracle."""
    s = layer.shape
    tok = ref["tokens"]
    rows = ref["row_of"].reshape(s.T, s.k)[tok]                      # [n_tok, k]
    h_gpu = G.bits_to_f64(out["h"][rows.reshape(-1)]).reshape(len(tok), s.k, s.F)
    yp_gpu = G.bits_to_f64(out["y_perm"][rows.reshape(-1)]).reshape(len(tok), s.k, s.d)
    y_gpu = G.bits_to_f64(out["y"][tok])
    e_h, e_v, e_y = _relmax(h_gpu, ref["h"]), _relmax(yp_gpu, ref["v"]), _relmax(y_gpu, ref["y"])
    _say(f"{s.name} T={s.T}: rel max err h={e_h:.2e} y_perm={e_v:.2e} y={e_y:.2e} "
         f"(max|y_ref|={np.abs(ref['y']).max():.3f})")
    assert np.isfinite(y_gpu).all()
    assert e_h <= REL and e_v <= REL and e_y <= REL
    return e_y


# ----------------------------------------------------------------------------- tiny, every stage
def test_tiny_whole_layer_and_stages(G):
    s = mi.PRESETS["tiny"]
    _say("tiny: moe_forward vs oracle")
    layer = G.Layer(s)
    ref = _oracle_full(layer)
    out = G.run_forward(layer)
    _check_routing(out, ref, layer)
    _check_floats(out, ref, layer, G)
    # determinism: a second run is bit-identical; row-major weights give the same integers and
    # floats within the tolerance (another kernel variant may sum over k in another order)
    out2 = G.run_forward(layer)
    out3 = G.run_forward(layer, packed=False)
    for key in out:
        assert np.array_equal(out[key], out2[key]), key
    _check_routing(out3, ref, layer)
    _check_floats(out3, ref, layer, G)
    # the packed buffer is a pure permutation of the three weight tensors
    pk = np.sort(G.np_bits(layer.packed.view(torch.bfloat16)).reshape(-1))
    raw = np.sort(np.concatenate([G.np_bits(t).reshape(-1) for t in (layer.wg, layer.wu, layer.wd)]))
    assert np.array_equal(pk, raw)
    # stage entry points one by one, fed with the ORACLE's upstream results
    idx, w = G.run_route(layer)
    assert np.array_equal(idx, ref["topk_idx"]) and np.abs(w - ref["topk_w"]).max() <= 1e-6
    cfg = layer.cfg()
    c, o, ro, so, xp = G.run_permute(cfg, ref["topk_idx"], layer.x)
    assert np.array_equal(c, ref["counts"]) and np.array_equal(o, ref["offsets"])
    assert np.array_equal(ro, ref["row_of"]) and np.array_equal(so, ref["src_of"])
    xp_ref = orc.permute_rows(layer.x_bits, ref["src_of"], s.k)
    assert np.array_equal(xp, xp_ref)
    rows = ref["row_of"].reshape(s.T, s.k)
    for packed in (True, False):
        h_bits, yp_bits = G.run_ffn(layer, cfg, xp_ref, ref["offsets"], packed=packed)
        assert _relmax(G.bits_to_f64(h_bits[rows]), ref["h"]) <= REL
        assert _relmax(G.bits_to_f64(yp_bits[rows]), ref["v"]) <= REL
    # combine fed with the oracle's FFN outputs rounded to bf16 (input prep, not method arithmetic)
    v_perm = np.zeros((s.R, s.d))
    v_perm[rows.reshape(-1)] = ref["v"].reshape(-1, s.d)
    vb = mi.bits(torch.from_numpy(v_perm).float().to(torch.bfloat16))
    y_bits = G.run_combine(cfg, vb, ref["row_of"], ref["topk_w"].astype(np.float32))
    y_ref = sum(ref["topk_w"].astype(np.float32).astype(np.float64)[:, i:i + 1] * G.bits_to_f64(vb[rows[:, i]])
                for i in range(s.k))
    assert _relmax(G.bits_to_f64(y_bits), y_ref) <= 2.0 ** -8


@pytest.mark.parametrize("packed", [True, False])
@pytest.mark.parametrize("tile_m", [32, 64, 96, 128, 160, 192, 256])
def test_ragged_shape_every_tile_height(G, tile_m, packed):
    """Rows per expert that are no multiple of any tile, feature dims with a ragged last
    feature tile (F=320, d=192), empty experts, and every GEMM variant."""
    s = mi.MoEShape("ragged", 333, 192, 320, 7, 3, mi.GATE_SOFTMAX_RENORM)
    _say(f"ragged T=333 d=192 F=320 E=7 k=3 tile_m={tile_m} packed={packed}")
    layer = G.Layer(s, seed=3, skew=2.0)          # strong skew: one expert holds ~T rows, some few
    ref = _oracle_full(layer)
    out = G.run_forward(layer, tile_m=tile_m, packed=packed)
    _check_routing(out, ref, layer)
    _check_floats(out, ref, layer, G)


@pytest.mark.parametrize("gating", [mi.GATE_SOFTMAX, mi.GATE_SOFTMAX_RENORM, mi.GATE_SIGMOID_NORM])
def test_many_experts_small_batches(G, gating):
    """E=256, k=8 (the DeepSeek-V3 routing shape) with narrow layers: most experts hold 0-3 rows."""
    s = mi.MoEShape("e256", 50, 128, 192, 256, 8, gating)
    _say(f"E=256 k=8 T=50 gating={gating}")
    layer = G.Layer(s, seed=5)
    ref = _oracle_full(layer)
    assert (ref["counts"] == 0).sum() > 20
    out = G.run_forward(layer)
    _check_routing(out, ref, layer)
    _check_floats(out, ref, layer, G)


@pytest.mark.parametrize("packed", [True, False])
@pytest.mark.parametrize("T,E,k", [(1, 8, 2), (2, 4, 4), (65, 1, 1), (1025, 3, 2)])
def test_degenerate_shapes(G, T, E, k, packed):
    """Single token, k == E (dense mixture), a single expert, and a token count that crosses the
    permutation kernels' 1024-slot chunk."""
    s = mi.MoEShape("edge", T, 64, 128, E, k, mi.GATE_SOFTMAX)
    _say(f"edge T={T} E={E} k={k}")
    layer = G.Layer(s, seed=7)
    ref = _oracle_full(layer)
    out = G.run_forward(layer, packed=packed)
    _check_routing(out, ref, layer)
    _check_floats(out, ref, layer, G)


@pytest.mark.parametrize("T,E", [(300, 8), (2100, 8), (700, 5), (300, 16)])
def test_router_paths_agree_with_the_oracle(G, T, E):
    """Few experts and few tokens take the single-kernel router, everything else the fp64-MFMA
    tiles + top-k kernel: both sides of each switch (E <= 8, T <= 2048), all three gatings."""
    for gating in (mi.GATE_SOFTMAX, mi.GATE_SOFTMAX_RENORM, mi.GATE_SIGMOID_NORM):
        s = mi.MoEShape("route", T, 320, 64, E, 2, gating)
        _say(f"router T={T} E={E} gating={gating}")
        layer = G.Layer(s, seed=21 + gating, skew=1.0)
        idx_ref, w_ref, gap = orc.route(layer.x_bits, layer.wr_bits, layer.bias_np, s.k, gating)
        assert gap.min() > GAP_MIN, "seeded logits too close to certify index parity"
        idx, w = G.run_route(layer)
        assert np.array_equal(idx, idx_ref)
        assert np.abs(w.astype(np.float64) - w_ref).max() <= 1e-6


@pytest.mark.parametrize("shape", [("a", 333, 192, 320, 7, 3), ("b", 1500, 256, 384, 4, 2)])
def test_forward_equals_the_stage_entry_points(G, shape):
    """moe_forward reads token rows through src_of inside the gate+up kernel; moe_permute +
    moe_grouped_ffn + moe_combine work on the materialised permuted copy.  Same kernels, same
    values, same order of summation: the bits of h, y_perm and y must be identical."""
    s = mi.MoEShape(*shape, mi.GATE_SOFTMAX_RENORM)
    _say(f"forward vs stages T={s.T} d={s.d} F={s.F} E={s.E} k={s.k}")
    layer = G.Layer(s, seed=5, skew=1.0)
    out = G.run_forward(layer)
    cfg = layer.cfg()
    idx, w = G.run_route(layer)
    c, o, ro, so, xp = G.run_permute(cfg, idx, layer.x)
    h_bits, yp_bits = G.run_ffn(layer, cfg, xp, o)
    y_bits = G.run_combine(cfg, yp_bits, ro, w)
    assert np.array_equal(idx, out["topk_idx"]) and np.array_equal(w, out["topk_w"])
    assert np.array_equal(ro, out["row_of"]) and np.array_equal(so, out["src_of"])
    assert np.array_equal(h_bits, out["h"])
    assert np.array_equal(yp_bits, out["y_perm"])
    assert np.array_equal(y_bits, out["y"])


def test_row_tiles_of_an_expert_side_by_side(G, monkeypatch):
    """Experts of three row tiles (two full, one short) on shapes whose feature-tile counts are
    multiples of 8, so that the default kernels re-order the workgroups inside each expert's span
    (row tiles that share a weight panel next to each other on one XCD): every element against the
    oracle, and bit-equal to the plain tile-major order and to Algorithm 1's row ranges (same
    per-row arithmetic, different workgroups)."""
    s = mi.MoEShape("three_tiles", 900, 2048, 2048, 3, 2, mi.GATE_SOFTMAX)
    layer = G.Layer(s, seed=11, skew=0.5)
    ref = _oracle_full(layer)
    assert (ref["counts"] > 512).any() and (ref["counts"] % 256 != 0).all()
    _say("three-tile experts, side-by-side launch order")
    out = G.run_forward(layer)
    _check_routing(out, ref, layer)
    _check_floats(out, ref, layer, G)
    monkeypatch.setenv("MOE_SIB", "0")
    _say("three-tile experts, tile-major launch order")
    plain = G.run_forward(layer)
    monkeypatch.delenv("MOE_SIB")
    for name in ("h", "y_perm", "y"):
        assert np.array_equal(out[name], plain[name]), name
    # the same for the row ranges: by default an expert of two or three row tiles has its rows
    # dealt evenly over them, MOE_EVEN=0 keeps Algorithm 1's ranges (256, 256, rest)
    monkeypatch.setenv("MOE_EVEN", "0")
    _say("three-tile experts, Algorithm 1's row ranges")
    alg1 = G.run_forward(layer)
    monkeypatch.delenv("MOE_EVEN")
    for name in ("h", "y_perm", "y"):
        assert np.array_equal(out[name], alg1[name]), name


def test_lds_dma_variants_and_graph_replay(G, monkeypatch):
    """The GEMM kernels that stage EVERY token tile with LDS-DMA loads (selected by environment
    variable; the default kernel uses that body only for experts spanning several row tiles)
    against the oracle, and a HIP-graph capture of moe_forward on the default path (one expert
    with two row tiles, the rest single blocks) whose replays must equal the eager result bit for
    bit (the library enqueues kernels only)."""
    import paper_2605_23911_amd as moe
    s = mi.MoEShape("ragged", 333, 192, 320, 7, 3, mi.GATE_SOFTMAX_RENORM)
    layer = G.Layer(s, seed=3, skew=2.0)
    ref = _oracle_full(layer)
    monkeypatch.setenv("MOE_GU_VARIANT", "3")
    monkeypatch.setenv("MOE_DN_VARIANT", "7")
    cfg = layer.cfg()
    assert "dma" in moe.ffn_kernel_name(cfg, 0, True) and "dma" in moe.ffn_kernel_name(cfg, 1, True)
    _say("LDS-DMA variants on the ragged shape")
    out = G.run_forward(layer)
    _check_routing(out, ref, layer)
    _check_floats(out, ref, layer, G)
    monkeypatch.delenv("MOE_GU_VARIANT")
    monkeypatch.delenv("MOE_DN_VARIANT")
    _say("graph capture + replays of the default path")
    lay = moe.forward_workspace_layout(cfg)
    ws = torch.zeros(lay.total, dtype=torch.uint8, device=G.DEV)
    y = torch.empty((s.T, s.d), dtype=torch.bfloat16, device=G.DEV)
    run = lambda: moe.moe_forward(cfg, layer.x, layer.wr, layer.bias, None, None, None, y, ws, W_packed=layer.packed)
    run()
    torch.cuda.synchronize()
    y_eager = y.clone()
    graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
    with torch.cuda.stream(side):
        run()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            run()
    for _ in range(3):
        y.zero_()
        ws.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, y_eager)
        run()                      # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(y, y_eager)


def test_zero_tokens_is_a_noop(G):
    import paper_2605_23911_amd as moe
    cfg = moe.MoEConfig.of(0, 64, 128, 4, 2)
    t = torch.zeros(4096, dtype=torch.uint8, device=G.DEV)
    moe.moe_forward(cfg, t, t, None, t, t, t, t, t, W_packed=t)
    torch.cuda.synchronize()
    assert int(t.sum().item()) == 0


# ----------------------------------------------------------------------------- integer stages at scale
@pytest.mark.parametrize("T,E,k,alpha", [(4096, 256, 8, 0.0), (4096, 64, 8, 2.0), (5000, 8, 2, 1.2), (37, 256, 8, 2.0)])
def test_permutation_and_schedule_bit_exact(G, T, E, k, alpha):
    """moe_permute / moe_block_schedule fed with injected assignments (the paper's Sec. 4.7
    methodology: Zipf-distributed experts), against the oracle's stable counting sort and Alg. 1."""
    import paper_2605_23911_amd as moe
    s = mi.MoEShape("perm", T, 64, 64, E, k)
    _say(f"permute T={T} E={E} k={k} zipf={alpha}")
    idx, _ = mi.zipf_assignments(s, alpha, seed=11)
    idx = idx.numpy()
    cfg = moe.MoEConfig.of(T, 64, 64, E, k)
    c_ref, o_ref, ro_ref, so_ref = orc.permutation(idx, E)
    x = mi.make_x(s, 11).to(G.DEV)
    c, o, ro, so, xp = G.run_permute(cfg, idx, x)
    assert np.array_equal(c, c_ref) and np.array_equal(o, o_ref)
    assert np.array_equal(ro, ro_ref) and np.array_equal(so, so_ref)
    assert np.array_equal(xp, orc.permute_rows(G.np_bits(x), so_ref, k))
    for M in (32, 64, 96, 160, 256):
        n, blocks, nmax = G.run_block_schedule(cfg, o_ref, M)
        want = orc.block_schedule(o_ref, M)
        assert n == len(want) <= nmax
        assert [tuple(b) for b in blocks.tolist()] == want


# ----------------------------------------------------------------------------- full-size configs, sampled rows
def _sampled_full_size(G, preset, T, n_tok, skew=0.0, packed=True):
    s = mi.PRESETS[preset].with_T(T)
    _say(f"{preset} T={T} skew={skew}: generating weights")
    layer = G.Layer(s, seed=0, skew=skew, keep_cpu_weights=False)
    _say(f"{preset} T={T}: moe_forward packed={packed}")
    out = G.run_forward(layer, packed=packed)
    _say(f"{preset} T={T}: oracle routing on all tokens, FFN on {n_tok} sampled tokens")
    idx_ref, _, _ = orc.route(layer.x_bits, layer.wr_bits, layer.bias_np, s.k, s.gating)
    counts = np.bincount(idx_ref.reshape(-1), minlength=s.E)
    hot = int(np.argmax(counts))
    cold = int(np.argmin(np.where(counts > 0, counts, counts.max() + 1)))
    rng = np.random.default_rng(1)
    tokens = set(rng.choice(T, size=min(n_tok, T), replace=False).tolist())
    tokens.add(int(np.nonzero((idx_ref == hot).any(axis=1))[0][0]))      # a row of the fullest expert
    tokens.add(int(np.nonzero((idx_ref == cold).any(axis=1))[0][-1]))    # and of the emptiest non-empty one
    ref = orc.moe_forward(layer.x_bits, layer.wr_bits, layer.bias_np, layer.expert_bits, s.k, s.gating,
                          tokens=sorted(tokens), keep_h=True)
    _check_routing(out, ref, layer)
    _check_floats(out, ref, layer, G)
    del layer
    torch.cuda.empty_cache()


def test_mixtral_T512_bench_configuration(G):
    _sampled_full_size(G, "mixtral", 512, 6)


def test_mixtral_T64_weight_bound_regime(G):
    _sampled_full_size(G, "mixtral", 64, 4)


def test_mixtral_T512_row_major_weights(G):
    _sampled_full_size(G, "mixtral", 512, 4, packed=False)


def test_mixtral_T4096_mfma_bound_regime(G):
    _sampled_full_size(G, "mixtral", 4096, 6)


def test_qwen2moe_T512_skewed(G):
    _sampled_full_size(G, "qwen2moe", 512, 6, skew=1.5)


def test_dsv3_T512(G):
    _sampled_full_size(G, "dsv3", 512, 3)


def test_mixtral_T1_decode(G):
    _sampled_full_size(G, "mixtral", 1, 1)


def test_qwen2moe_T4096(G):
    _sampled_full_size(G, "qwen2moe", 4096, 4)


def test_dsv3_T4096_skewed(G):
    """Skew 1 at the largest shape: a few experts hold thousands of rows (sixteen 256-row tiles:
    cached weights, k in step, tiles side by side), most a handful (one short block each:
    weights streamed once), all in one launch."""
    _sampled_full_size(G, "dsv3", 4096, 3, skew=1.0)
