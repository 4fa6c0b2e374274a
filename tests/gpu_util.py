"""Helpers for the GPU parity tests: seeded inputs on the device, stage runners that call the
C ABI through the binding, and numpy views of results.  Holds none of the method's arithmetic."""
from __future__ import annotations

import numpy as np
import torch

import moe_inputs as mi
import paper_2605_23911_amd as moe

DEV = "cuda:0"


def np_bits(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor on any device -> uint16 numpy bit patterns."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def bits_to_f64(u16: np.ndarray) -> np.ndarray:
    return (u16.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


class Bank:
    """The expert weights of one layer shape (they depend on d, F, E and the seed, not on T or
    the routing skew): device tensors, the one-time packed copy, and optionally the CPU bit
    patterns.  Several Layer objects (different T, different skew) can share one bank."""

    def __init__(self, shape: mi.MoEShape, seed: int = 0, keep_cpu_weights: bool = True):
        self.shape = shape
        self.seed = seed
        s = shape
        self.wg = torch.empty((s.E, s.F, s.d), dtype=torch.bfloat16, device=DEV)
        self.wu = torch.empty((s.E, s.F, s.d), dtype=torch.bfloat16, device=DEV)
        self.wd = torch.empty((s.E, s.d, s.F), dtype=torch.bfloat16, device=DEV)
        self._cpu_w = {} if keep_cpu_weights else None
        if keep_cpu_weights:
            for e in range(s.E):
                w = mi.make_expert(s, e, seed)
                self._cpu_w[e] = w
                self.wg[e].copy_(w[0]); self.wu[e].copy_(w[1]); self.wd[e].copy_(w[2])
        else:
            mi.make_all_experts(s, seed, out=(self.wg, self.wu, self.wd))
        # one-time packed copy of the expert weights (what a serving stack does at load time)
        cfg = moe.MoEConfig.of(1, s.d, s.F, s.E, s.k, s.gating)
        self.packed = torch.empty(moe.packed_weights_size(cfg), dtype=torch.uint8, device=DEV)
        moe.moe_pack_weights(cfg, self.wg, self.wu, self.wd, self.packed)
        torch.cuda.synchronize()

    def expert_bits(self, e: int):
        """Oracle-side weight provider: regenerates the expert from its seed when not cached."""
        w = self._cpu_w[e] if self._cpu_w is not None else mi.make_expert(self.shape, e, self.seed)
        return tuple(mi.bits(t) for t in w)


class Layer:
    """One seeded layer: CPU bit patterns for the oracle and device tensors for the library."""

    def __init__(self, shape: mi.MoEShape, seed: int = 0, skew: float = 0.0, keep_cpu_weights: bool = True,
                 bank: Bank | None = None):
        self.shape = shape
        self.seed = seed
        self.x_cpu = mi.make_x(shape, seed)
        self.wr_cpu = mi.make_router(shape, seed)
        self.bias_cpu = mi.skew_bias(shape, skew, seed)
        self.x = self.x_cpu.to(DEV)
        self.wr = self.wr_cpu.to(DEV)
        self.bias = None if self.bias_cpu is None else self.bias_cpu.to(DEV)
        if bank is None:
            bank = Bank(shape, seed, keep_cpu_weights)
        else:
            b = bank.shape
            assert (b.d, b.F, b.E, b.k, b.gating, bank.seed) == (shape.d, shape.F, shape.E, shape.k, shape.gating, seed)
        self.bank = bank
        self.wg, self.wu, self.wd, self.packed = bank.wg, bank.wu, bank.wd, bank.packed

    def cfg(self, tile_m: int = 0, T: int | None = None, flags: int = 0):
        s = self.shape
        return moe.MoEConfig.of(s.T if T is None else T, s.d, s.F, s.E, s.k, s.gating, tile_m, flags)

    def expert_bits(self, e: int):
        return self.bank.expert_bits(e)

    @property
    def x_bits(self):
        return mi.bits(self.x_cpu)

    @property
    def wr_bits(self):
        return mi.bits(self.wr_cpu)

    @property
    def bias_np(self):
        return None if self.bias_cpu is None else self.bias_cpu.numpy()


def run_forward(layer: Layer, tile_m: int = 0, packed: bool = True, flags: int = 0):
    """moe_forward through the C ABI; returns y bits and every intermediate from the workspace.
    packed=True hands the kernels the pre-packed weight copy only (row-major pointers NULL)."""
    cfg = layer.cfg(tile_m, flags=flags)
    s = layer.shape
    lay = moe.forward_workspace_layout(cfg)
    ws = torch.zeros(lay.total, dtype=torch.uint8, device=DEV)
    y = torch.empty((s.T, s.d), dtype=torch.bfloat16, device=DEV)
    if packed:
        moe.moe_forward(cfg, layer.x, layer.wr, layer.bias, None, None, None, y, ws, W_packed=layer.packed)
    else:
        moe.moe_forward(cfg, layer.x, layer.wr, layer.bias, layer.wg, layer.wu, layer.wd, y, ws)
    torch.cuda.synchronize()
    R = s.R

    def view(off, n, dt):
        return ws[off: off + n * torch.tensor([], dtype=dt).element_size()].view(dt)

    out = dict(
        y=np_bits(y),
        topk_idx=view(lay.topk_idx, R, torch.int32).cpu().numpy().reshape(s.T, s.k),
        topk_w=view(lay.topk_w, R, torch.float32).cpu().numpy().reshape(s.T, s.k),
        counts=view(lay.counts, s.E, torch.int32).cpu().numpy(),
        offsets=view(lay.offsets, s.E + 1, torch.int32).cpu().numpy(),
        row_of=view(lay.row_of, R, torch.int32).cpu().numpy(),
        src_of=view(lay.src_of, R, torch.int32).cpu().numpy(),
        h=np_bits(view(lay.h, R * s.F, torch.bfloat16)).reshape(R, s.F),
        y_perm=np_bits(view(lay.y_perm, R * s.d, torch.bfloat16)).reshape(R, s.d),
    )
    return out


def run_route(layer: Layer):
    cfg = layer.cfg()
    s = layer.shape
    idx = torch.full((s.T, s.k), -7, dtype=torch.int32, device=DEV)
    w = torch.zeros((s.T, s.k), dtype=torch.float32, device=DEV)
    ws = torch.zeros(max(moe.route_workspace_size(cfg), 256), dtype=torch.uint8, device=DEV)
    moe.moe_route(cfg, layer.x, layer.wr, layer.bias, idx, w, ws)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), w.cpu().numpy()


def run_permute(cfg, topk_idx: np.ndarray, x: torch.Tensor | None):
    T, k, E, d = cfg.T, cfg.k, cfg.E, cfg.d
    R = T * k
    idx = torch.from_numpy(np.ascontiguousarray(topk_idx, dtype=np.int32)).to(DEV)
    counts = torch.full((E,), -1, dtype=torch.int32, device=DEV)
    offsets = torch.full((E + 1,), -1, dtype=torch.int32, device=DEV)
    row_of = torch.full((max(R, 1),), -1, dtype=torch.int32, device=DEV)
    src_of = torch.full((max(R, 1),), -1, dtype=torch.int32, device=DEV)
    x_perm = None if x is None else torch.zeros((max(R, 1), d), dtype=torch.bfloat16, device=DEV)
    ws = torch.zeros(max(moe.permute_workspace_size(cfg), 256), dtype=torch.uint8, device=DEV)
    moe.moe_permute(cfg, x, idx, counts, offsets, row_of, src_of, x_perm, ws)
    torch.cuda.synchronize()
    return (counts.cpu().numpy(), offsets.cpu().numpy(), row_of.cpu().numpy()[:R], src_of.cpu().numpy()[:R],
            None if x is None else np_bits(x_perm)[:R])


def run_block_schedule(cfg, offsets: np.ndarray, M: int):
    off = torch.from_numpy(np.ascontiguousarray(offsets, dtype=np.int32)).to(DEV)
    nmax = moe.max_blocks(cfg, M)
    blocks = torch.full((max(nmax, 1), 2), -1, dtype=torch.int32, device=DEV)
    nb = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    moe.moe_block_schedule(cfg, off, M, blocks, nb)
    torch.cuda.synchronize()
    n = int(nb.item())
    return n, blocks.cpu().numpy()[:n], nmax


def run_ffn(layer: Layer, cfg, x_perm_bits: np.ndarray, offsets: np.ndarray, packed: bool = True):
    s = layer.shape
    R = cfg.T * cfg.k
    xp = torch.from_numpy(x_perm_bits.view(np.int16).copy()).view(torch.bfloat16).to(DEV)
    off = torch.from_numpy(np.ascontiguousarray(offsets, dtype=np.int32)).to(DEV)
    h = torch.zeros((R, s.F), dtype=torch.bfloat16, device=DEV)
    yp = torch.zeros((R, s.d), dtype=torch.bfloat16, device=DEV)
    ws = torch.zeros(moe.ffn_workspace_size(cfg), dtype=torch.uint8, device=DEV)
    if packed:
        moe.moe_grouped_ffn(cfg, xp, off, None, None, None, h, yp, ws, W_packed=layer.packed)
    else:
        moe.moe_grouped_ffn(cfg, xp, off, layer.wg, layer.wu, layer.wd, h, yp, ws)
    torch.cuda.synchronize()
    return np_bits(h), np_bits(yp)


def run_combine(cfg, y_perm_bits: np.ndarray, row_of: np.ndarray, topk_w: np.ndarray):
    yp = torch.from_numpy(y_perm_bits.view(np.int16).copy()).view(torch.bfloat16).to(DEV)
    ro = torch.from_numpy(np.ascontiguousarray(row_of, dtype=np.int32)).to(DEV)
    w = torch.from_numpy(np.ascontiguousarray(topk_w, dtype=np.float32)).to(DEV)
    y = torch.zeros((cfg.T, cfg.d), dtype=torch.bfloat16, device=DEV)
    moe.moe_combine(cfg, yp, ro, w, y)
    torch.cuda.synchronize()
    return np_bits(y)
