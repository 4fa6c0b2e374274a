"""CPU oracle for one MoE layer's forward pass.  TEST INFRASTRUCTURE ONLY.

Plain numpy, fp64, written from the paper's equations (Sec. 2.1, Eq. 1-4), the
block-schedule listing (Sec. 3.2, Algorithm 1) and the router / permutation
descriptions (Sec. 3.4, 3.5).  It shares no code with the HIP path and must never
be imported by the product package: only tests, the smoke check and the
benchmark's `cpu_baseline` leg call it.

Inputs are the *bit patterns* of bf16 tensors (numpy uint16); they are decoded
exactly to fp64 and nothing is rounded afterwards.  The layer output `y` is
computed token by token straight from Eq. 3-4; the permutation (Sec. 3.5) is
computed separately as its own checked result and is NOT used to produce `y`.

Readings taken where the paper is silent (they are listed in the design notes):
  * top-k selects on the logits z (softmax is strictly increasing, so in exact
    arithmetic this is the same set and order as selecting on the scores);
    ties go to the lower expert index; outputs are in selection order.
  * weights are the raw softmax scores (Eq. 2-3) unless `gating` asks for the
    renormalised or the sigmoid form (Sec. 3.4, last sentence).
  * SiLU(a) = a / (1 + exp(-a)).
  * stored weights are [out, in] (reduction dim contiguous, Sec. 3.2 "E*N x K"),
    so Eq. 4's  x W  is  x @ W.T  of the stored matrix.

Pins (tests/test_oracle_pins.py): softmax closed forms, brute-force sort for
top-k and the tie rule, numpy bincount/cumsum/stable argsort for the permutation,
Algorithm 1 worked by hand, E=1,k=1 dense SwiGLU, all-experts-identical = dense
FFN, k=E full mixture, an independent pure-Python scalar evaluation of the
whole layer, linearity and token-permutation equivariance.
"""
from __future__ import annotations

import numpy as np

GATE_SOFTMAX = 0
GATE_SOFTMAX_RENORM = 1
GATE_SIGMOID_NORM = 2


def bf16_to_f64(u16: np.ndarray) -> np.ndarray:
    """Exact value of bf16 bit patterns: bf16 is the top half of an IEEE fp32."""
    u16 = np.ascontiguousarray(u16, dtype=np.uint16)
    return (u16.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


# --------------------------------------------------------------------------- #
# Routing: Eq. 1 (scores), Eq. 2 (top-k), Sec. 3.4
# --------------------------------------------------------------------------- #
def router_logits(x_bits, wr_bits, bias=None) -> np.ndarray:
    """z[t, e] = sum_i x[t, i] * W_r[e, i] (+ b[e]).  Argument of Eq. 1's softmax."""
    z = bf16_to_f64(x_bits) @ bf16_to_f64(wr_bits).T
    if bias is not None:
        z = z + np.asarray(bias, dtype=np.float32).astype(np.float64)[None, :]
    return z


def softmax_rows(z: np.ndarray) -> np.ndarray:
    """Eq. 1 with the row maximum subtracted first (Sec. 3.4)."""
    ez = np.exp(z - z.max(axis=1, keepdims=True))
    return ez / ez.sum(axis=1, keepdims=True)


def topk_select(z: np.ndarray, k: int) -> np.ndarray:
    """Eq. 2 as Sec. 3.4 describes it: k rounds of argmax, each winner masked out.

    numpy's argmax returns the first maximum, i.e. the lower index on a tie."""
    T, E = z.shape
    assert 1 <= k <= E
    work = z.copy()
    idx = np.empty((T, k), dtype=np.int32)
    rows = np.arange(T)
    for i in range(k):
        win = np.argmax(work, axis=1)
        idx[:, i] = win
        work[rows, win] = -np.inf
    return idx


def topk_min_gap(z: np.ndarray, k: int) -> np.ndarray:
    """Per token: smallest difference between neighbours among the k+1 largest
    logits (k largest when k == E).  A gap far above fp64 summation error
    certifies that any fp64 summation order selects the same experts in the
    same order."""
    T, E = z.shape
    srt = -np.sort(-z, axis=1)[:, : min(k + 1, E)]
    if srt.shape[1] < 2:
        return np.full(T, np.inf)
    return (srt[:, :-1] - srt[:, 1:]).min(axis=1)


def gate_weights(z: np.ndarray, idx: np.ndarray, gating: int) -> np.ndarray:
    """w_i of Eq. 2 for the selected experts."""
    rows = np.arange(z.shape[0])[:, None]
    if gating == GATE_SIGMOID_NORM:
        sg = 1.0 / (1.0 + np.exp(-z[rows, idx]))
        return sg / sg.sum(axis=1, keepdims=True)
    w = softmax_rows(z)[rows, idx]
    if gating == GATE_SOFTMAX_RENORM:
        w = w / w.sum(axis=1, keepdims=True)
    elif gating != GATE_SOFTMAX:
        raise ValueError("unknown gating")
    return w


def route(x_bits, wr_bits, bias, k: int, gating: int):
    """(topk_idx int32 [T,k], topk_w fp64 [T,k], min_gap fp64 [T])."""
    z = router_logits(x_bits, wr_bits, bias)
    idx = topk_select(z, k)
    return idx, gate_weights(z, idx, gating), topk_min_gap(z, k)


# --------------------------------------------------------------------------- #
# Permutation into expert-contiguous order: Sec. 2.2 (n_e), Sec. 3.5
# --------------------------------------------------------------------------- #
def permutation(topk_idx: np.ndarray, E: int):
    """Stable sort of the flat slot list j = t*k + i by expert id.

    counts[e] = n_e; offsets = exclusive prefix sum (offsets[E] = T*k);
    row_of[j] = destination row of slot j; src_of[r] = slot stored at row r."""
    flat = np.asarray(topk_idx, dtype=np.int64).reshape(-1)
    counts = np.zeros(E, dtype=np.int32)
    for e in flat:
        counts[e] += 1
    offsets = np.zeros(E + 1, dtype=np.int32)
    for e in range(E):
        offsets[e + 1] = offsets[e] + counts[e]
    cursor = offsets[:-1].copy()
    row_of = np.empty(flat.size, dtype=np.int32)
    src_of = np.empty(flat.size, dtype=np.int32)
    for j, e in enumerate(flat):
        r = cursor[e]
        cursor[e] += 1
        row_of[j] = r
        src_of[r] = j
    return counts, offsets, row_of, src_of


def permute_rows(x_bits: np.ndarray, src_of: np.ndarray, k: int) -> np.ndarray:
    """x_perm[r, :] = x[src_of[r] // k, :]  (a copy of bit patterns)."""
    return np.asarray(x_bits)[np.asarray(src_of) // k]


def block_schedule(offsets, M: int):
    """Sec. 3.2's block schedule (Algorithm 1): expert by expert, the row offsets 0, M, 2M, ...
    below n_e, each paired with the expert id; an expert without rows contributes nothing."""
    return [(e, r) for e in range(len(offsets) - 1)
            for r in range(0, int(offsets[e + 1]) - int(offsets[e]), M)]


# --------------------------------------------------------------------------- #
# Expert FFN (Eq. 4) and combine (Eq. 3)
# --------------------------------------------------------------------------- #
def silu(a: np.ndarray) -> np.ndarray:
    return a / (1.0 + np.exp(-a))


def expert_ffn(xrows: np.ndarray, wg_bits, wu_bits, wd_bits):
    """Eq. 4 for the rows of `xrows` (fp64 [n, d]) through one expert.

    Returns (h [n, F], v [n, d]): the SwiGLU intermediate and FFN_e(x)."""
    wg = bf16_to_f64(wg_bits)
    g = xrows @ wg.T
    del wg
    wu = bf16_to_f64(wu_bits)
    u = xrows @ wu.T
    del wu
    h = silu(g) * u
    wd = bf16_to_f64(wd_bits)
    v = h @ wd.T
    return h, v


def moe_forward(x_bits, wr_bits, bias, expert_weights, k: int, gating: int,
                tokens=None, topk=None, keep_h: bool = False):
    """Whole layer, Eq. 1-4.

    expert_weights(e) -> (W_gate[e] [F,d], W_up[e] [F,d], W_down[e] [d,F]) bit patterns.
    tokens: optional list of token ids; the FFN (the costly part) is evaluated for
        these only.  Routing and the permutation always cover every token.
    topk: optional precomputed (topk_idx, topk_w) replacing the router (Sec. 4.7's
        methodology of injecting assignments).

    Returns a dict with topk_idx, topk_w, min_gap, counts, offsets, row_of, src_of,
    tokens, v [n_tok, k, d] (FFN_{e_i}(x_t)), y [n_tok, d], and h [n_tok, k, F] if keep_h.
    """
    x_bits = np.asarray(x_bits)
    T, d = x_bits.shape
    E = np.asarray(wr_bits).shape[0]
    if topk is None:
        idx, w, gap = route(x_bits, wr_bits, bias, k, gating)
    else:
        idx = np.asarray(topk[0], dtype=np.int32)
        w = np.asarray(topk[1]).astype(np.float64)
        gap = np.full(T, np.inf)
    counts, offsets, row_of, src_of = permutation(idx, E)

    tok = np.arange(T) if tokens is None else np.asarray(sorted(tokens), dtype=np.int64)
    x64 = bf16_to_f64(x_bits[tok])
    v = np.zeros((tok.size, k, d), dtype=np.float64)
    h_all = None
    # FFN_{e_i}(x_t) for every selected (t, i).  The loop runs over experts only so
    # that each expert's weights are decoded once; every (t, i) is still evaluated
    # independently as a row of a plain matrix product.
    for e in range(E):
        tt, ii = np.nonzero(idx[tok] == e)
        if tt.size == 0:
            continue
        wg, wu, wd = expert_weights(e)
        h, ve = expert_ffn(x64[tt], wg, wu, wd)
        v[tt, ii] = ve
        if keep_h:
            if h_all is None:
                h_all = np.zeros((tok.size, k, h.shape[1]), dtype=np.float64)
            h_all[tt, ii] = h
    # Eq. 3: weighted sum over the selected experts, in slot order.
    y = np.zeros((tok.size, d), dtype=np.float64)
    for i in range(k):
        y += w[tok, i][:, None] * v[:, i, :]
    out = dict(topk_idx=idx, topk_w=w, min_gap=gap, counts=counts, offsets=offsets,
               row_of=row_of, src_of=src_of, tokens=tok, v=v, y=y)
    if keep_h:
        out["h"] = h_all
    return out
