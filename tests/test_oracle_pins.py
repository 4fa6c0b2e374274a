"""Pins for the CPU oracle: closed forms, library routines, brute force, and an
independent scalar pure-Python evaluation of Eq. 1-4.  No GPU, no HIP code."""
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

import moe_inputs as mi
from oracle import moe_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _bits(a: np.ndarray) -> np.ndarray:
    """float array -> bf16 bit patterns through torch's RNE conversion."""
    return mi.bits(torch.from_numpy(np.asarray(a, dtype=np.float32)).to(torch.bfloat16))


def _val(b: np.ndarray) -> np.ndarray:
    """Independent bf16 decode (torch) used to cross-check the oracle's own."""
    t = torch.from_numpy(b.view(np.int16).copy()).view(torch.bfloat16)
    return t.double().numpy()


def _rand_layer(T, d, F, E, seed=0):
    rng = np.random.default_rng(seed)
    x = _bits(rng.standard_normal((T, d)))
    wr = _bits(rng.standard_normal((E, d)) / math.sqrt(d))
    wg = _bits(rng.standard_normal((E, F, d)) / math.sqrt(d))
    wu = _bits(rng.standard_normal((E, F, d)) / math.sqrt(d))
    wd = _bits(rng.standard_normal((E, d, F)) / math.sqrt(F))
    return x, wr, wg, wu, wd


def _provider(wg, wu, wd):
    return lambda e: (wg[e], wu[e], wd[e])


# ------------------------------------------------------------------ bf16 decode
def test_bf16_decode_known_patterns():
    pats = np.array([0x3F80, 0xC000, 0x0000, 0x8000, 0x3DCD, 0x0001, 0x7F7F, 0x4049], np.uint16)
    want = [1.0, -2.0, 0.0, -0.0, 0.10009765625, 2.0 ** -133, (2 - 2 ** -7) * 2.0 ** 127, 3.140625]
    got = orc.bf16_to_f64(pats)
    assert got.tolist() == want
    assert math.copysign(1.0, got[3]) == -1.0
    rnd = np.random.default_rng(1).integers(0, 0x7F80, 4096).astype(np.uint16)
    assert np.array_equal(orc.bf16_to_f64(rnd), _val(rnd))


# ------------------------------------------------------------------ softmax
def test_softmax_closed_forms():
    rng = np.random.default_rng(2)
    z = rng.standard_normal((37, 19)) * 5
    s = orc.softmax_rows(z)
    assert np.abs(s.sum(axis=1) - 1).max() < 1e-14
    assert np.abs(orc.softmax_rows(z + 123.25) - s).max() < 1e-13
    assert np.abs(s - scipy.special.softmax(z, axis=1)).max() < 1e-15
    assert np.all(orc.softmax_rows(np.zeros((3, 8))) == 0.125)
    # huge logits must not overflow (the reason Sec. 3.4 gives for subtracting the max)
    big = np.array([[1000.0, 999.0, -1000.0]])
    e = math.exp(-1.0)
    assert np.allclose(orc.softmax_rows(big)[0], [1 / (1 + e), e / (1 + e), 0.0], atol=1e-15)


def test_router_logits_match_scalar_sum_and_bias():
    x, wr, *_ = _rand_layer(6, 24, 8, 5, seed=3)
    bias = np.linspace(-1, 1, 5).astype(np.float32)
    z = orc.router_logits(x, wr, bias)
    xv, wv = _val(x), _val(wr)
    for t in range(6):
        for e in range(5):
            want = math.fsum(float(xv[t, i]) * float(wv[e, i]) for i in range(24)) + float(bias[e])
            assert abs(z[t, e] - want) < 1e-13
    # a transposed operand would fail here: z is [T, E]
    assert z.shape == (6, 5)


# ------------------------------------------------------------------ top-k
def test_topk_equals_bruteforce_sort():
    rng = np.random.default_rng(4)
    z = rng.standard_normal((200, 64))
    z[::7, 5] = z[::7, 40]            # planted exact ties
    z[::11, 63] = z[::11, 0]
    for k in (1, 2, 8, 64):
        got = orc.topk_select(z, k)
        for t in range(z.shape[0]):
            want = sorted(range(64), key=lambda e: (-z[t, e], e))[:k]
            assert got[t].tolist() == want


def test_topk_tie_rule_lower_index_and_zero_router():
    x, wr, *_ = _rand_layer(9, 16, 8, 8, seed=5)
    zero = np.zeros_like(wr)
    idx, w, gap = orc.route(x, zero, None, 3, orc.GATE_SOFTMAX)
    assert np.array_equal(idx, np.tile(np.arange(3, dtype=np.int32), (9, 1)))
    assert np.all(w == 0.125) and np.all(gap == 0)
    _, wn, _ = orc.route(x, zero, None, 3, orc.GATE_SOFTMAX_RENORM)
    assert np.allclose(wn, 1 / 3, atol=1e-16)
    # duplicated router rows a < b: whenever both are selected a comes right before b,
    # and b is never selected without a
    wr2 = wr.copy()
    wr2[6] = wr2[2]
    idx, w, _ = orc.route(x, wr2, None, 4, orc.GATE_SOFTMAX)
    for t in range(9):
        row = idx[t].tolist()
        if 6 in row:
            assert 2 in row and row.index(2) + 1 == row.index(6)
            assert w[t, row.index(2)] == w[t, row.index(6)]


def test_topk_order_is_descending_and_weights_are_scores():
    x, wr, *_ = _rand_layer(50, 32, 8, 16, seed=6)
    idx, w, gap = orc.route(x, wr, None, 4, orc.GATE_SOFTMAX)
    z = orc.router_logits(x, wr)
    s = scipy.special.softmax(z, axis=1)
    assert np.all(np.diff(w, axis=1) <= 0)
    assert np.abs(w - np.take_along_axis(s, idx.astype(np.int64), 1)).max() < 1e-15
    assert np.all(gap > 0)
    # min_gap against its definition
    for t in range(50):
        srt = sorted(z[t], reverse=True)[:5]
        assert gap[t] == pytest.approx(min(a - b for a, b in zip(srt, srt[1:])), abs=1e-15)


def test_gating_variants():
    x, wr, *_ = _rand_layer(40, 32, 8, 16, seed=7)
    z = orc.router_logits(x, wr)
    idx = orc.topk_select(z, 4)
    zs = np.take_along_axis(z, idx.astype(np.int64), 1)
    wn = orc.gate_weights(z, idx, orc.GATE_SOFTMAX_RENORM)
    assert np.abs(wn.sum(axis=1) - 1).max() < 1e-15
    assert np.abs(wn - scipy.special.softmax(zs, axis=1)).max() < 1e-14   # renorm == softmax over the k logits
    wsig = orc.gate_weights(z, idx, orc.GATE_SIGMOID_NORM)
    sg = scipy.special.expit(zs)
    assert np.abs(wsig - sg / sg.sum(axis=1, keepdims=True)).max() < 1e-15
    assert np.allclose(orc.gate_weights(np.zeros((2, 8)), np.array([[0, 1], [2, 3]]), orc.GATE_SIGMOID_NORM), 0.5)


# ------------------------------------------------------------------ permutation
@pytest.mark.parametrize("T,k,E", [(1, 1, 1), (1, 2, 8), (64, 2, 8), (300, 8, 256), (257, 3, 5)])
def test_permutation_against_numpy_routines(T, k, E):
    rng = np.random.default_rng(T * 131 + E)
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    counts, offsets, row_of, src_of = orc.permutation(idx, E)
    flat = idx.reshape(-1)
    assert np.array_equal(counts, np.bincount(flat, minlength=E))
    assert counts.sum() == T * k and offsets[0] == 0 and offsets[E] == T * k
    assert np.array_equal(offsets[1:], np.cumsum(counts))
    assert np.array_equal(src_of, np.argsort(flat, kind="stable"))
    assert np.array_equal(row_of[src_of], np.arange(T * k))
    assert np.array_equal(src_of[row_of], np.arange(T * k))
    for e in range(E):
        seg = src_of[offsets[e]:offsets[e + 1]]
        assert np.all(flat[seg] == e) and np.all(np.diff(seg) > 0)
    # permute then unpermute returns every token's row k times
    x = rng.integers(0, 65536, (T, 6)).astype(np.uint16)
    xp = orc.permute_rows(x, src_of, k)
    assert np.array_equal(xp[row_of].reshape(T, k, 6), np.repeat(x[:, None, :], k, axis=1))


def test_block_schedule_golden_and_properties():
    lines = [l for l in open(os.path.join(GOLD, "alg1_block_schedule.txt")) if not l.startswith("#")]
    want = [tuple(int(v) for v in l.split()) for l in lines if l.strip()]
    assert orc.block_schedule([0, 5, 5, 6, 14], 4) == want
    rng = np.random.default_rng(8)
    for M in (1, 16, 64, 128):
        n = rng.integers(0, 300, 40)
        n[rng.integers(0, 40, 10)] = 0
        off = np.concatenate([[0], np.cumsum(n)])
        blocks = orc.block_schedule(off, M)
        assert len(blocks) == sum(-(-int(v) // M) for v in n)
        covered = np.zeros(off[-1], dtype=int)
        for e, r0 in blocks:
            assert n[e] > 0 and r0 % M == 0 and r0 < n[e]
            covered[off[e] + r0: off[e] + min(r0 + M, n[e])] += 1
        assert np.all(covered == 1)
        assert blocks == sorted(blocks)


def test_golden_table1_and_launch_counts():
    rows = {}
    for l in open(os.path.join(GOLD, "table1_model_shapes.txt")):
        if not l.startswith("#"):
            n, E, k, d, F = l.split()
            rows[n] = (int(E), int(k), int(d), int(F))
    for preset, name in (("mixtral", "Mixtral-8x7B"), ("mixtral22", "Mixtral-8x22B"), ("dsv3", "DeepSeek-V3")):
        s = mi.PRESETS[preset]
        assert (s.E, s.k, s.d, s.F) == rows[name]
    q = mi.PRESETS["qwen2moe"]            # top-k 8 by the benchmark contract, 4 in Table 1
    assert (q.E, q.d, q.F) == (rows["Qwen2-MoE-57B"][0],) + rows["Qwen2-MoE-57B"][2:]
    for l in open(os.path.join(GOLD, "launch_counts.txt")):
        if not l.startswith("#"):
            E, gemms, total, ours = (int(v) for v in l.split())
            assert gemms == 3 * E and total == 3 * E + 4 and ours == 5


# ------------------------------------------------------------------ FFN / whole layer
def test_single_expert_is_dense_swiglu_against_torch():
    x, wr, wg, wu, wd = _rand_layer(7, 48, 80, 1, seed=9)
    out = orc.moe_forward(x, wr, None, _provider(wg, wu, wd), 1, orc.GATE_SOFTMAX, keep_h=True)
    assert np.all(out["topk_idx"] == 0) and np.all(out["topk_w"] == 1.0)
    tx = torch.from_numpy(_val(x))
    g = tx @ torch.from_numpy(_val(wg[0])).T
    u = tx @ torch.from_numpy(_val(wu[0])).T
    h = torch.nn.functional.silu(g) * u
    y = h @ torch.from_numpy(_val(wd[0])).T
    assert np.abs(out["h"][:, 0] - h.numpy()).max() < 1e-13
    assert np.abs(out["y"] - y.numpy()).max() < 1e-13
    assert np.abs(out["y"]).max() > 0.05


def _python_layer(x, wr, wg, wu, wd, bias, k, gating):
    """Eq. 1-4 with Python floats and loops only; written apart from the oracle."""
    T, d = len(x), len(x[0])
    E, F = len(wg), len(wg[0])
    ys, picks = [], []
    for t in range(T):
        z = [sum(x[t][i] * wr[e][i] for i in range(d)) + (bias[e] if bias is not None else 0.0)
             for e in range(E)]
        m = max(z)
        ex = [math.exp(v - m) for v in z]
        s = [v / sum(ex) for v in ex]
        order = sorted(range(E), key=lambda e: (-z[e], e))[:k]
        if gating == orc.GATE_SOFTMAX:
            w = [s[e] for e in order]
        elif gating == orc.GATE_SOFTMAX_RENORM:
            tot = sum(s[e] for e in order)
            w = [s[e] / tot for e in order]
        else:
            sg = [1 / (1 + math.exp(-z[e])) for e in order]
            w = [v / sum(sg) for v in sg]
        y = [0.0] * d
        for e, we in zip(order, w):
            hvec = []
            for f in range(F):
                g = sum(x[t][i] * wg[e][f][i] for i in range(d))
                u = sum(x[t][i] * wu[e][f][i] for i in range(d))
                hvec.append(g / (1 + math.exp(-g)) * u)
            for c in range(d):
                y[c] += we * sum(hvec[f] * wd[e][c][f] for f in range(F))
        ys.append(y)
        picks.append((order, w))
    return ys, picks


@pytest.mark.parametrize("gating", [orc.GATE_SOFTMAX, orc.GATE_SOFTMAX_RENORM, orc.GATE_SIGMOID_NORM])
@pytest.mark.parametrize("use_bias", [False, True])
def test_whole_layer_against_pure_python(gating, use_bias):
    T, d, F, E, k = 5, 8, 6, 4, 2
    x, wr, wg, wu, wd = _rand_layer(T, d, F, E, seed=10 + gating)
    bias = np.array([0.5, -1.0, 0.25, 0.0], np.float32) if use_bias else None
    out = orc.moe_forward(x, wr, bias, _provider(wg, wu, wd), k, gating)
    ys, picks = _python_layer(_val(x).tolist(), _val(wr).tolist(), _val(wg).tolist(), _val(wu).tolist(),
                              _val(wd).tolist(), None if bias is None else bias.tolist(), k, gating)
    for t in range(T):
        assert out["topk_idx"][t].tolist() == picks[t][0]
        assert np.abs(out["topk_w"][t] - np.array(picks[t][1])).max() < 1e-14
    assert np.abs(out["y"] - np.array(ys)).max() < 1e-12
    assert np.abs(out["y"]).max() > 1e-3


def test_whole_layer_against_pure_python_square_matrices():
    """E = d = F: every weight matrix is square, the one case in which a transposed operand
    multiplies without a shape error."""
    T, n, k = 4, 6, 3
    x, wr, wg, wu, wd = _rand_layer(T, n, n, n, seed=17)
    out = orc.moe_forward(x, wr, None, _provider(wg, wu, wd), k, orc.GATE_SOFTMAX_RENORM)
    ys, picks = _python_layer(_val(x).tolist(), _val(wr).tolist(), _val(wg).tolist(), _val(wu).tolist(),
                              _val(wd).tolist(), None, k, orc.GATE_SOFTMAX_RENORM)
    for t in range(T):
        assert out["topk_idx"][t].tolist() == picks[t][0]
        assert np.abs(out["topk_w"][t] - np.array(picks[t][1])).max() < 1e-14
    assert np.abs(out["y"] - np.array(ys)).max() < 1e-12
    assert np.abs(out["y"]).max() > 1e-3


def test_layer_invariants():
    T, d, F, E, k = 12, 32, 40, 6, 3
    x, wr, wg, wu, wd = _rand_layer(T, d, F, E, seed=20)
    base = orc.moe_forward(x, wr, None, _provider(wg, wu, wd), k, orc.GATE_SOFTMAX)
    # SiLU(0) = 0: zero gate weights give zero output
    z = orc.moe_forward(x, wr, None, _provider(np.zeros_like(wg), wu, wd), k, orc.GATE_SOFTMAX)
    assert np.all(z["y"] == 0)
    # linear in W_down: doubling it (exact in bf16) doubles y exactly
    wd2 = _bits(2.0 * _val(wd))
    dbl = orc.moe_forward(x, wr, None, _provider(wg, wu, wd2), k, orc.GATE_SOFTMAX)
    assert np.array_equal(dbl["y"], 2.0 * base["y"])
    # token-permutation equivariance
    p = np.random.default_rng(21).permutation(T)
    per = orc.moe_forward(x[p], wr, None, _provider(wg, wu, wd), k, orc.GATE_SOFTMAX)
    assert np.array_equal(per["topk_idx"], base["topk_idx"][p])
    assert np.abs(per["y"] - base["y"][p]).max() < 1e-13
    # all experts identical + renormalised weights = dense FFN whatever the routing
    same = lambda a: np.repeat(a[:1], E, axis=0)
    ident = orc.moe_forward(x, wr, None, _provider(same(wg), same(wu), same(wd)), k, orc.GATE_SOFTMAX_RENORM)
    _, dense = orc.expert_ffn(_val(x), wg[0], wu[0], wd[0])
    assert np.abs(ident["y"] - dense).max() < 1e-13
    # k = E without renormalisation = full softmax mixture of all experts
    full = orc.moe_forward(x, wr, None, _provider(wg, wu, wd), E, orc.GATE_SOFTMAX)
    s = scipy.special.softmax(orc.router_logits(x, wr), axis=1)
    mix = sum(s[:, e:e + 1] * orc.expert_ffn(_val(x), wg[e], wu[e], wd[e])[1] for e in range(E))
    assert np.abs(full["y"] - mix).max() < 1e-13
    # a token subset gives the same rows as the full evaluation
    sub = orc.moe_forward(x, wr, None, _provider(wg, wu, wd), k, orc.GATE_SOFTMAX, tokens=[7, 2, 11])
    assert sub["tokens"].tolist() == [2, 7, 11]
    assert np.abs(sub["y"] - base["y"][[2, 7, 11]]).max() < 1e-13
    # injected assignments (Sec. 4.7's methodology) bypass the router
    inj = orc.moe_forward(x, wr, None, _provider(wg, wu, wd), k, orc.GATE_SOFTMAX,
                          topk=(base["topk_idx"], base["topk_w"]))
    assert np.abs(inj["y"] - base["y"]).max() < 1e-13


@pytest.mark.parametrize("d,F,c,f", [(8, 16, 5, 11), (16, 16, 5, 11)])
def test_down_projection_is_not_transposed(d, F, c, f):
    # a W_down [d, F] with a single non-zero entry at (c, f): y[:, c] = h[:, f] * w.  With d != F a
    # transposed operand cannot even be multiplied; with d == F it can, silently, hence both shapes.
    T = 3
    x, wr, wg, wu, wd = _rand_layer(T, d, F, 1, seed=22)
    wd0 = np.zeros((1, d, F), np.float32)
    wd0[0, c, f] = 3.0
    out = orc.moe_forward(x, wr, None, _provider(wg, wu, _bits(wd0)), 1, orc.GATE_SOFTMAX, keep_h=True)
    want = np.zeros((T, d))
    want[:, c] = 3.0 * out["h"][:, 0, f]
    assert np.array_equal(out["y"], want)


# ------------------------------------------------------------------ input recipe
def test_inputs_are_seeded_and_scaled():
    s = mi.PRESETS["tiny"]
    a, b = mi.make_x(s, 0), mi.make_x(s, 0)
    assert torch.equal(a, b) and not torch.equal(a, mi.make_x(s, 1))
    wg, wu, wd = mi.make_expert(s, 3, 0)
    assert wg.shape == (s.F, s.d) and wd.shape == (s.d, s.F) and not torch.equal(wg, wu)
    assert abs(wg.float().std().item() * math.sqrt(s.d) - 1) < 0.05
    assert abs(wd.float().std().item() * math.sqrt(s.F) - 1) < 0.05
    allw = mi.make_all_experts(s, 0, threads=2)
    assert torch.equal(allw[0][3], wg) and torch.equal(allw[2][3], wd)
    bias = mi.skew_bias(mi.PRESETS["qwen2moe"], 1.5, 0)
    p = np.exp(bias.double().numpy())
    assert abs(p.sum() - 1) < 1e-5 and np.isclose(np.sort(p)[-1] / np.sort(p)[-2], 2 ** 1.5, rtol=1e-5)
    assert mi.skew_bias(s, 0.0) is None
    idx, w = mi.zipf_assignments(s, 1.2, 0)
    assert idx.shape == (s.T, s.k) and all(len(set(r.tolist())) == s.k for r in idx)


def test_tiny_config_routing_is_certified():
    """On the seeded tiny config the top-(k+1) logit gaps are far above fp64 noise."""
    s = mi.PRESETS["tiny"]
    idx, w, gap = orc.route(mi.bits(mi.make_x(s)), mi.bits(mi.make_router(s)), None, s.k, s.gating)
    assert gap.min() > 1e-9
    counts = orc.permutation(idx, s.E)[0]
    assert counts.sum() == s.T * s.k and counts.min() > 0
