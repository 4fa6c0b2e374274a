"""Seeded synthetic inputs for one MoE layer (shapes of Table 1 of the paper).

This module only draws random numbers and rounds them to bf16.  It holds none of
the method's arithmetic and is the only code that both the CPU oracle's tests and
the HIP path's tests/bench use: the same bf16 bit patterns go to both sides.

Recipe (every tensor is rounded to bf16, round-to-nearest-even, by torch):
    x              ~ N(0, 1)        [T, d]
    W_r            ~ N(0, 1/d)      [E, d]
    W_gate, W_up   ~ N(0, 1/d)      [E, F, d]   (reduction dim contiguous)
    W_down         ~ N(0, 1/F)      [E, d, F]   (reduction dim contiguous)
With these scales the router logits are ~N(0,1), which gives the near-uniform
routing the paper benchmarks on (its Sec. 4.7, first paragraph).  Routing skew is
injected as a per-expert logit bias log(p_e), p_e ~ 1/rank^s over a seeded random
ranking of the experts.

Every tensor (and every expert of the expert weights) has its own generator
stream, derived from (seed, tensor id, expert), so one expert's weights can be
regenerated without materialising the other experts.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
import math
import os

import numpy as np
import torch

GATE_SOFTMAX = 0          # w_i = softmax(z)[e_i]                       (Eq. 1-2)
GATE_SOFTMAX_RENORM = 1   # w_i = softmax(z)[e_i] / sum_j softmax(z)[e_j]
GATE_SIGMOID_NORM = 2     # w_i = sigmoid(z_{e_i}) / sum_j sigmoid(z_{e_j})  (Sec. 3.4)

_X, _WR, _WG, _WU, _WD, _RANK, _TIE = range(7)


@dataclass(frozen=True)
class MoEShape:
    name: str
    T: int
    d: int
    F: int
    E: int
    k: int
    gating: int = GATE_SOFTMAX

    @property
    def R(self) -> int:
        return self.T * self.k

    def with_T(self, T: int) -> "MoEShape":
        return replace(self, T=T)


# Table 1 of the paper, with the top-k of the benchmark contract for Qwen2-MoE (8).
PRESETS = {
    "tiny":     MoEShape("tiny", 64, 256, 512, 8, 2, GATE_SOFTMAX),
    "mixtral":  MoEShape("mixtral", 512, 4096, 14336, 8, 2, GATE_SOFTMAX),
    "qwen2moe": MoEShape("qwen2moe", 512, 3584, 2560, 64, 8, GATE_SOFTMAX_RENORM),
    "dsv3":     MoEShape("dsv3", 512, 7168, 2048, 256, 8, GATE_SOFTMAX),
    "mixtral22": MoEShape("mixtral22", 512, 6144, 16384, 8, 2, GATE_SOFTMAX),
}


def _gen(seed: int, tensor_id: int, expert: int = 0) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed((seed * 1_000_003 + tensor_id) * 4099 + expert)
    return g


def _normal_bf16(shape, std: float, g: torch.Generator) -> torch.Tensor:
    t = torch.randn(shape, generator=g, dtype=torch.float32)
    if std != 1.0:
        t.mul_(std)
    return t.to(torch.bfloat16)


def bits(t: torch.Tensor) -> np.ndarray:
    """bf16 torch tensor (CPU) -> uint16 numpy array of the same bit patterns."""
    assert t.dtype == torch.bfloat16 and t.device.type == "cpu"
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def make_x(s: MoEShape, seed: int = 0) -> torch.Tensor:
    return _normal_bf16((s.T, s.d), 1.0, _gen(seed, _X))


def make_router(s: MoEShape, seed: int = 0) -> torch.Tensor:
    return _normal_bf16((s.E, s.d), 1.0 / math.sqrt(s.d), _gen(seed, _WR))


def make_expert(s: MoEShape, e: int, seed: int = 0):
    """(W_gate[e] [F,d], W_up[e] [F,d], W_down[e] [d,F]) as bf16 CPU tensors."""
    wg = _normal_bf16((s.F, s.d), 1.0 / math.sqrt(s.d), _gen(seed, _WG, e))
    wu = _normal_bf16((s.F, s.d), 1.0 / math.sqrt(s.d), _gen(seed, _WU, e))
    wd = _normal_bf16((s.d, s.F), 1.0 / math.sqrt(s.F), _gen(seed, _WD, e))
    return wg, wu, wd


def make_all_experts(s: MoEShape, seed: int = 0, out=None, threads: int | None = None):
    """All expert weights, generated expert by expert on a thread pool.

    `out`, if given, is a triple of preallocated bf16 tensors ([E,F,d], [E,F,d],
    [E,d,F]) on any device that the experts are copied into as they are made.
    """
    if out is None:
        out = (torch.empty((s.E, s.F, s.d), dtype=torch.bfloat16),
               torch.empty((s.E, s.F, s.d), dtype=torch.bfloat16),
               torch.empty((s.E, s.d, s.F), dtype=torch.bfloat16))
    threads = threads or min(16, os.cpu_count() or 1)

    def one(e):
        return e, make_expert(s, e, seed)

    with ThreadPoolExecutor(max_workers=threads) as pool:
        for e, (wg, wu, wd) in pool.map(one, range(s.E)):
            out[0][e].copy_(wg)
            out[1][e].copy_(wu)
            out[2][e].copy_(wd)
    return out


def skew_bias(s: MoEShape, skew: float, seed: int = 0):
    """fp32 logit bias log(p_e), p_e = rank_e^-skew / sum; None when skew == 0."""
    if skew == 0.0:
        return None
    perm = torch.randperm(s.E, generator=_gen(seed, _RANK)).numpy()
    rank = np.empty(s.E, dtype=np.float64)
    rank[perm] = np.arange(1, s.E + 1, dtype=np.float64)
    p = rank ** (-float(skew))
    p /= p.sum()
    return torch.from_numpy(np.log(p).astype(np.float32))


def zipf_assignments(s: MoEShape, alpha: float, seed: int = 0):
    """Precomputed (indices, weights) in the manner of the paper's Sec. 4.7: each
    token draws k distinct experts with probability ~ 1/rank^alpha (alpha = 0 is
    uniform); weights are 1/k.  Feeds moe_permute onward, bypassing the router."""
    g = _gen(seed, _TIE)
    p = torch.arange(1, s.E + 1, dtype=torch.float64) ** (-float(alpha))
    p = (p / p.sum()).expand(s.T, s.E)
    idx = torch.multinomial(p, s.k, replacement=False, generator=g).to(torch.int32)
    w = torch.full((s.T, s.k), 1.0 / s.k, dtype=torch.float32)
    return idx, w
