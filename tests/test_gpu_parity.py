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


@pytest.mark.parametrize("T,E,k,d", [(255, 16, 2, 320), (256, 16, 2, 320), (300, 40, 4, 320), (700, 100, 8, 448),
                                      (512, 256, 8, 1024)])
def test_router_first_pass_and_exact_candidates(G, knobs, T, E, k, d):
    """For large batches (here: forced from 256 tokens on) the router computes all logits on the bf16 matrix cores first and
    recomputes only the experts within the error bound of the k-th largest in fp64: the same
    indices in the same order as the oracle, weights within 1e-6, on one, two and four 32-expert
    tiles per wavefront with ragged last tiles, all three gatings; and the same indices as the
    all-fp64 path (255 tokens take that path by themselves)."""
    import paper_2605_23911_amd.binding as B
    for gating in (mi.GATE_SOFTMAX, mi.GATE_SOFTMAX_RENORM, mi.GATE_SIGMOID_NORM):
        s = mi.MoEShape("route2", T, d, 64, E, k, gating)
        _say(f"router T={T} E={E} k={k} d={d} gating={gating}")
        layer = G.Layer(s, seed=31 + gating, skew=1.0)
        idx_ref, w_ref, gap = orc.route(layer.x_bits, layer.wr_bits, layer.bias_np, s.k, gating)
        assert gap.min() > GAP_MIN, "seeded logits too close to certify index parity"
        knobs(B.KNOB_ROUTE_EXACT, 0)     # the first pass from 256 tokens on (by itself: from 2^19 logits on)
        idx, w = G.run_route(layer)
        assert np.array_equal(idx, idx_ref)
        assert np.abs(w.astype(np.float64) - w_ref).max() <= 1e-6
        knobs(B.KNOB_ROUTE_EXACT, 1)
        idx2, w2 = G.run_route(layer)
        knobs(B.KNOB_ROUTE_EXACT, -1)
        assert np.array_equal(idx2, idx_ref)
        assert np.abs(w2.astype(np.float64) - w.astype(np.float64)).max() <= 3e-7


def test_router_ties_on_the_first_pass_path(G, knobs):
    """Exact ties, where the first pass cannot tell experts apart: duplicated router rows (the
    lower index must win, both at the selection boundary and inside the selected set) and an
    all-zero router (every expert is a candidate: experts 0..k-1, weights 1/E)."""
    import paper_2605_23911_amd.binding as B
    knobs(B.KNOB_ROUTE_EXACT, 0)
    s = mi.MoEShape("ties", 300, 320, 64, 70, 4, mi.GATE_SOFTMAX)
    layer = G.Layer(s, seed=5)
    wr = layer.wr_cpu.clone()
    wr[9] = wr[2]
    wr[69] = wr[0]
    wr[33] = wr[34]
    layer.wr_cpu = wr
    layer.wr = wr.to(G.DEV)
    idx_ref, w_ref, _ = orc.route(layer.x_bits, layer.wr_bits, None, s.k, s.gating)
    idx, w = G.run_route(layer)
    assert np.array_equal(idx, idx_ref)
    assert np.abs(w.astype(np.float64) - w_ref).max() <= 1e-6
    both = ((idx == 2).any(axis=1) & (idx == 9).any(axis=1)).sum(), ((idx == 2).any(axis=1) ^ (idx == 9).any(axis=1)).sum()
    assert both[0] > 0 and both[1] > 0, "the duplicated pair should appear both inside the top-k and across its boundary"
    layer.wr_cpu = torch.zeros_like(wr)
    layer.wr = layer.wr_cpu.to(G.DEV)
    idx, w = G.run_route(layer)
    assert np.array_equal(idx, np.tile(np.arange(s.k, dtype=np.int32), (s.T, 1)))
    assert np.abs(w - 1.0 / s.E).max() <= 1e-7


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


@pytest.fixture
def knobs():
    """Sets test knobs of the library for one test and restores the selection rules afterwards."""
    import paper_2605_23911_amd.binding as B
    touched = []

    def set_knob(which, value):
        touched.append(which)
        B.test_knob(which, value)

    yield set_knob
    for which in touched:
        B.test_knob(which, -1)


def _all_rows_against_oracle(G, layer, ref, out):
    """Every element of h, y_perm and y against the full oracle; no row left unwritten."""
    _check_routing(out, ref, layer)
    _check_floats(out, ref, layer, G)
    assert (out["h"] != 0).any(axis=1).all(), "a row of h was never written"
    assert (out["y_perm"] != 0).any(axis=1).all(), "a row of y_perm was never written"


def test_row_tiles_of_an_expert_side_by_side(G, knobs):
    """Experts of three row tiles (two full, one short) on shapes whose feature-tile counts are
    multiples of 8, so that the default kernels re-order the workgroups inside each expert's span
    (row tiles that share a weight panel next to each other on one XCD): every element against the
    oracle, and bit-equal to the plain tile-major order and to Algorithm 1's row ranges (same
    per-row arithmetic, different workgroups)."""
    import paper_2605_23911_amd.binding as B
    s = mi.MoEShape("three_tiles", 900, 2048, 2048, 3, 2, mi.GATE_SOFTMAX)
    layer = G.Layer(s, seed=11, skew=0.5)
    ref = _oracle_full(layer)
    assert (ref["counts"] > 512).any() and (ref["counts"] % 256 != 0).all()
    _say("three-tile experts, side-by-side launch order")
    out = G.run_forward(layer)
    _all_rows_against_oracle(G, layer, ref, out)
    knobs(B.KNOB_SIDE_BY_SIDE, 0)
    _say("three-tile experts, tile-major launch order")
    plain = G.run_forward(layer)
    knobs(B.KNOB_SIDE_BY_SIDE, -1)
    for name in ("h", "y_perm", "y"):
        assert np.array_equal(out[name], plain[name]), name
    # the same for the row ranges: by default an expert of two or three row tiles has its rows
    # dealt evenly over them; knob 0 keeps Algorithm 1's ranges (256, 256, rest)
    knobs(B.KNOB_EVEN_ROWS, 0)
    _say("three-tile experts, Algorithm 1's row ranges")
    alg1 = G.run_forward(layer)
    for name in ("h", "y_perm", "y"):
        assert np.array_equal(out[name], alg1[name]), name


# Shapes for the launch orders of multi-tile experts, all rows checked.  d = 2048 and F = 1024
# give feature-tile counts that are multiples of 8 for both projections (F/128 = 8; d/128 = 16,
# d/256 = 8), which is what switches the side-by-side order on.
#   five_tiles : 2 experts x 1100 rows = 4 full tiles + 76 rows.  gate+up: side by side with the
#                short tile moved to the end of the span (n = 5, n - 1 tiles in step).  down: 80
#                two-block workgroups are at most half a round, so each is split into two
#                128-feature halves.
#   nine_tiles : 2 experts x 2100 rows = 8 full tiles + 52 rows.  Both projections side by side
#                with the short tile at the end; the down projection in its two-weight-block form.
#   skewed16   : 16 experts under skew 2: one of 4 full tiles + a short one, one of three tiles,
#                one of two, the rest single blocks or empty, in one launch.  down: single-use
#                weights, one contiguous eighth of the work per XCD.
#   mixed8, mixed12 : three multi-tile experts (8, 5 and 2-3 tiles) and five / nine single-block
#                ones with many rows per expert on average, which is where the down projection
#                deals its heavy and light blocks evenly over the launch: block by block with
#                d/256 = 7 feature tiles (mixed8), in units of 8 workgroups with 8 (mixed12).
_TILE_SHAPES = {
    "five_tiles": (mi.MoEShape("five_tiles", 1100, 2048, 1024, 2, 2, mi.GATE_SOFTMAX), 11, 0.0),
    "nine_tiles": (mi.MoEShape("nine_tiles", 2100, 2048, 1024, 2, 2, mi.GATE_SOFTMAX_RENORM), 12, 0.0),
    "skewed16": (mi.MoEShape("skewed16", 1090, 2048, 1024, 16, 2, mi.GATE_SOFTMAX), 11, 2.0),
    "mixed8": (mi.MoEShape("mixed8", 2000, 1792, 1024, 8, 2, mi.GATE_SOFTMAX), 11, 2.0),
    "mixed12": (mi.MoEShape("mixed12", 2000, 2048, 1024, 12, 2, mi.GATE_SOFTMAX), 12, 2.0),
    # feature-tile counts that are no multiples of 8 (10 for gate+up, 6 for the down projection): the
    # side-by-side order then leaves some panels' row tiles spread over several XCDs
    "odd_tiles": (mi.MoEShape("odd_tiles", 1600, 1536, 1280, 3, 2, mi.GATE_SOFTMAX), 11, 0.0),
}


@pytest.mark.parametrize("name", sorted(_TILE_SHAPES))
def test_multi_tile_experts_all_rows(G, knobs, name):
    """Experts of four and more row tiles with a short last one, every element of h, y_perm and
    y against the oracle, in each launch order the kernels have: side by side with the short
    tile at the end of the span, a last round split in halves, per-XCD chunks; then bit-equal
    results with each re-ordering switched off and with the rows dealt evenly."""
    import paper_2605_23911_amd as moe
    import paper_2605_23911_amd.binding as B
    s, seed, skew = _TILE_SHAPES[name]
    layer = G.Layer(s, seed=seed, skew=skew)
    ref = _oracle_full(layer)
    hot = int(ref["counts"].max())
    assert hot > 4 * 256 and (name.startswith("mixed") or 0 < hot % 256 <= 96), "the fullest expert must end in a short tile"
    cfg = layer.cfg()
    if name == "five_tiles":
        assert moe.ffn_kernel_name(cfg, 1, True).startswith("tile_kernel_mixed<2, false, true, false")
    if name == "skewed16":
        assert moe.ffn_kernel_name(cfg, 1, True).startswith("tile_kernel_mixed<1, false, true, true")
        assert sorted(ref["counts"])[-2] > 512 and sorted(ref["counts"])[-3] > 256
    if name.startswith("mixed"):
        assert moe.ffn_kernel_name(cfg, 1, True).startswith("tile_kernel_mixed<2, false, true, false")
        assert (ref["counts"] > 256).sum() == 3 and ((ref["counts"] > 0) & (ref["counts"] <= 256)).sum() >= 5
    _say(f"{name}: default launch order, all rows")
    out = G.run_forward(layer)
    _all_rows_against_oracle(G, layer, ref, out)
    # Which workgroup computes a row does not change the row's result as long as k is walked in
    # the same order.  By default a short last tile of a multi-tile expert walks k rotated (it
    # streams its panel like a single-block expert); for the bit-for-bit comparisons below that
    # is switched off, so that a row gives the same bits whichever tile it falls into.
    knobs(B.KNOB_SHORT_NT, 0)
    _say(f"{name}: short tiles in step with their siblings, all rows")
    out = G.run_forward(layer)
    _all_rows_against_oracle(G, layer, ref, out)
    for which, value, label in [(B.KNOB_SIDE_BY_SIDE, 0, "tile-major order"), (B.KNOB_EVEN_ROWS, 0, "Algorithm 1's row ranges"),
                                (B.KNOB_EVEN_ROWS, 3, "rows dealt evenly everywhere")]:
        knobs(which, value)
        _say(f"{name}: {label}")
        other = G.run_forward(layer)
        knobs(which, -1)
        for key in ("h", "y_perm", "y"):
            assert np.array_equal(out[key], other[key]), (label, key)
    # The per-XCD chunking changes which workgroup id computes a block, and single-block experts
    # start their k loop at a step that depends on the id: another order of the same sum, so
    # these two are compared with the oracle, not bit for bit.
    # The same holds for the dealing of heavy and light blocks over the down projection's launch.
    for which, value, label in [(B.KNOB_XCD_CHUNK, 0, "no per-XCD chunks"), (B.KNOB_XCD_CHUNK, 1, "per-XCD chunks on both projections"),
                                (B.KNOB_INTERLEAVE, 0, "down projection in expert order"),
                                (B.KNOB_INTERLEAVE, 1, "heavy and light blocks dealt whatever their proportion")]:
        knobs(which, value)
        _say(f"{name}: {label}")
        other = G.run_forward(layer)
        knobs(which, -1)
        _all_rows_against_oracle(G, layer, ref, other)


def test_expert_span_across_a_split_last_round(G, knobs):
    """Down projection with two weight blocks per wavefront whose launch is one full round of the
    CUs plus a last round at most half full (that round's tiles are split into 128-feature halves),
    with an expert of seven row tiles whose span lies partly in the full round and partly in the
    split one: 3 experts x ~1667 rows, d = 4096 -> 21 blocks x 16 tiles = 336 workgroups on 256 CUs,
    spans [0,112) [112,224) [224,336).  Every element against the oracle, and bit-equal with the
    side-by-side order off; the same launch is enumerated on the host as well."""
    import torch
    import paper_2605_23911_amd as moe
    import paper_2605_23911_amd.binding as B
    s = mi.MoEShape("straddle", 5000, 4096, 1024, 3, 1, mi.GATE_SOFTMAX)
    layer = G.Layer(s, seed=13, skew=0.0)
    ref = _oracle_full(layer)
    cfg = layer.cfg()
    assert moe.tile_m(cfg) == 256 and moe.ffn_kernel_name(cfg, 1, True).startswith("tile_kernel_mixed<2, false, true, false")
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    tiles = [(int(c) + 255) // 256 * (s.d // 256) for c in ref["counts"]]
    total, ends = sum(tiles), np.cumsum(tiles)
    assert cus < total <= cus + cus // 2, "the launch must be one full round and a last round at most half full"
    assert cus not in ends and min(tiles) >= 2 * (s.d // 256), "a multi-tile expert's span must cross the round boundary"
    offsets = ref["offsets"].astype(np.int32)
    blocks = np.array(orc.block_schedule(offsets, 256), dtype=np.int32)
    work = B.map_launch(False, 2, False, s.d, 256, offsets, blocks, cus=cus, slack_blocks=moe.max_blocks(cfg, 256) - len(blocks))
    cover = np.zeros((s.R, s.d // 128), dtype=np.int16)
    for has, e, row0, rows, nt, width in work:
        if has:
            cover[row0:row0 + rows, nt * width:(nt + 1) * width] += 1
    assert cover.min() == 1 and cover.max() == 1 and (work[:, 5] == 1).sum() == 2 * (total - cus)
    knobs(B.KNOB_SHORT_NT, 0)    # every tile walks k from step 0: bit-for-bit comparisons below
    _say("straddle: default launch order, all rows")
    out = G.run_forward(layer)
    _all_rows_against_oracle(G, layer, ref, out)
    knobs(B.KNOB_SIDE_BY_SIDE, 0)
    _say("straddle: tile-major order")
    plain = G.run_forward(layer)
    for key in ("h", "y_perm", "y"):
        assert np.array_equal(out[key], plain[key]), key


@pytest.mark.parametrize("shape,skew", [(("ragged", 333, 192, 320, 7, 3), 2.0), (("wide", 700, 512, 256, 16, 4), 1.0),
                                        (("five_tiles", 1100, 2048, 1024, 2, 2), 0.0), (("e256", 300, 256, 192, 256, 8), 0.0)])
def test_combine_folded_into_the_down_projection(G, shape, skew):
    """moe_forward lets the down-projection workgroup that writes the last of a token's k rows
    form y (no separate combine launch).  The sum is taken in slot order from the bf16 rows in
    memory whoever arrives last, so y must be bit-equal to the separate combine kernel's (knob 0),
    identical from run to run, and within tolerance of the oracle."""
    s = mi.MoEShape(*shape, mi.GATE_SOFTMAX_RENORM)
    layer = G.Layer(s, seed=9, skew=skew)
    ref = _oracle_full(layer)
    import paper_2605_23911_amd as moe
    _say(f"{s.name}: combine folded into the down projection (MOE_FLAG_FUSE_COMBINE)")
    fused = [G.run_forward(layer, flags=moe.FLAG_FUSE_COMBINE) for _ in range(3)]
    _say(f"{s.name}: separate combine launch")
    plain = G.run_forward(layer)
    _check_routing(fused[0], ref, layer)
    _check_floats(fused[0], ref, layer, G)
    for out in fused:
        for key in ("h", "y_perm", "y"):
            assert np.array_equal(out[key], plain[key]), key


def test_down_projection_variants_and_graph_replay(G, knobs):
    """Every packed down-projection kernel forced onto the ragged shape (the selection rules
    would pick only one of them at this size) against the oracle, and a HIP-graph capture of
    moe_forward on the default path (one expert with two row tiles, the rest single blocks)
    whose replays must equal the eager result bit for bit (the library enqueues kernels only)."""
    import paper_2605_23911_amd as moe
    import paper_2605_23911_amd.binding as B
    s = mi.MoEShape("ragged", 333, 192, 320, 7, 3, mi.GATE_SOFTMAX_RENORM)
    layer = G.Layer(s, seed=3, skew=2.0)
    ref = _oracle_full(layer)
    cfg = layer.cfg()
    for variant, frag in [(5, "mixed<1, false, true, true"), (6, "mixed<2, false, true, true"), (7, "mixed<2, false, true, false")]:
        knobs(B.KNOB_DOWN_VARIANT, variant)
        assert frag in moe.ffn_kernel_name(cfg, 1, True)
        _say(f"down-projection variant {variant} on the ragged shape")
        out = G.run_forward(layer)
        _all_rows_against_oracle(G, layer, ref, out)
    knobs(B.KNOB_DOWN_VARIANT, -1)
    for flags, label in [(0, "default path"), (moe.FLAG_FUSE_COMBINE, "combine folded into the down projection")]:
        _say(f"graph capture + replays: {label}")
        cfg = layer.cfg(flags=flags)
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
            ws.fill_(0xff if flags else 0)   # the layer must clear its own arrival counters
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(y, y_eager)
            run()                      # eager work between the replays
            torch.cuda.synchronize()
            assert torch.equal(y, y_eager)


@pytest.mark.parametrize("skew", [0.0, 2.0])
def test_two_workgroups_per_cu(G, knobs, skew):
    """Many experts with few rows each at up to 128 tokens: blocks of at most 128 rows and the GEMM
    kernels built for two workgroups per CU.  Chosen by the rule on a 256-expert shape (uniform
    routing: 3 rows per expert; skewed: one expert holds most tokens, the four-block body), and
    forced onto the ragged shape; every element against the oracle, bit-equal with the combine
    folded in."""
    import paper_2605_23911_amd as moe
    import paper_2605_23911_amd.binding as B
    s = mi.MoEShape("many_small", 100, 1024, 256, 256, 8, mi.GATE_SOFTMAX)
    layer = G.Layer(s, seed=9, skew=skew)
    cfg = layer.cfg()
    assert moe.tile_m(cfg) == 128
    assert moe.ffn_kernel_name(cfg, 0, True) == "tile_kernel_mixed<1, true, true, true, true>"
    assert moe.ffn_kernel_name(cfg, 1, True) == "tile_kernel_mixed<1, false, true, true, true>"
    beyond = moe.MoEConfig.of(129, s.d, s.F, s.E, s.k, s.gating)     # 129 tokens: the one-workgroup-per-CU kernels
    assert moe.tile_m(beyond) == 256 and "true, true, true>" not in moe.ffn_kernel_name(beyond, 1, True)
    ref = _oracle_full(layer)
    if skew > 0:
        assert ref["counts"].max() > 64
    _say(f"two workgroups per CU by rule, skew {skew}: all rows")
    out = G.run_forward(layer)
    _all_rows_against_oracle(G, layer, ref, out)
    fused = G.run_forward(layer, flags=moe.FLAG_FUSE_COMBINE)
    for key in ("h", "y_perm", "y"):
        assert np.array_equal(out[key], fused[key]), key
    # forced: ragged shape, blocks of 128 rows (experts of up to ~300 rows: several blocks each)
    r = mi.MoEShape("ragged", 333, 192, 320, 7, 3, mi.GATE_SOFTMAX_RENORM)
    rl = G.Layer(r, seed=3, skew=skew)
    rref = _oracle_full(rl)
    knobs(B.KNOB_GATE_UP_VARIANT, 2)
    knobs(B.KNOB_DOWN_VARIANT, 8)
    assert moe.ffn_kernel_name(rl.cfg(128), 1, True) == "tile_kernel_mixed<1, false, true, true, true>"
    _say(f"two workgroups per CU forced onto the ragged shape, skew {skew}")
    out = G.run_forward(rl, tile_m=128)
    _all_rows_against_oracle(G, rl, rref, out)


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


# The full-size configurations of the benchmark contract (every T of every shape, the skew grid,
# the second workload sweep) are in test_gpu_contract_cells.py.
