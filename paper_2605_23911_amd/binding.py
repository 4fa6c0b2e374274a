"""ctypes binding of include/moe.h: argument marshalling only.

Tensors are torch tensors on the GPU (torch is used for device memory and streams only);
their data pointers and the current stream handle are passed straight to the C ABI.
"""
from __future__ import annotations

import ctypes as C
import os

import torch  # imported before the library so that both share one HIP runtime

GATE_SOFTMAX = 0
GATE_SOFTMAX_RENORM = 1
GATE_SIGMOID_NORM = 2
FLAG_FUSE_COMBINE = 1

_LIB_NAME = "libmoe_mi355x.so"
_lib = None

EXPORTS = (
    "moe_status_string", "moe_tile_m", "moe_route_workspace_size", "moe_permute_workspace_size", "moe_ffn_workspace_size",
    "moe_forward_workspace_size", "moe_workspace_size", "moe_forward_workspace_layout", "moe_max_blocks", "moe_route",
    "moe_permute", "moe_permute_static", "moe_block_schedule", "moe_grouped_ffn", "moe_combine", "moe_forward", "moe_forward_staged", "moe_packed_weights_size", "moe_pack_weights", "moe_ffn_kernel_name",
)


class MoEError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().moe_status_string(status).decode() if _lib is not None else str(status)
        super().__init__(f"{where}: {msg} (status {status})")


class MoEConfig(C.Structure):
    _fields_ = [("T", C.c_int32), ("d", C.c_int32), ("F", C.c_int32), ("E", C.c_int32), ("k", C.c_int32),
                ("gating", C.c_int32), ("tile_m", C.c_int32), ("flags", C.c_int32)]

    @classmethod
    def of(cls, T, d, F, E, k, gating=GATE_SOFTMAX, tile_m=0, flags=0):
        return cls(T, d, F, E, k, gating, tile_m, flags)


class WorkspaceLayout(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("topk_idx", "topk_w", "counts", "offsets", "row_of", "src_of",
                                          "x_perm", "h", "y_perm", "scratch", "total")]


def library_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), _LIB_NAME)


def lib() -> C.CDLL:
    """Load the HIP library (built in-tree by build.py).  No fallback: raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with `python -m paper_2605_23911_amd.build` "
                           "(or __graft_entry__.build()); there is no CPU fallback")
    L = C.CDLL(path)
    cfgp, vp, i32p, f32p = C.POINTER(MoEConfig), C.c_void_p, C.c_void_p, C.c_void_p
    L.moe_status_string.restype = C.c_char_p
    L.moe_status_string.argtypes = [C.c_int]
    L.moe_ffn_kernel_name.restype = C.c_char_p
    L.moe_ffn_kernel_name.argtypes = [cfgp, C.c_int32, C.c_int32]
    L.moe_tile_m.restype = C.c_int32
    L.moe_tile_m.argtypes = [cfgp]
    L.moe_max_blocks.restype = C.c_int32
    L.moe_max_blocks.argtypes = [cfgp, C.c_int32]
    for n in ("moe_route_workspace_size", "moe_permute_workspace_size", "moe_ffn_workspace_size", "moe_forward_workspace_size",
              "moe_workspace_size", "moe_packed_weights_size"):
        getattr(L, n).restype = C.c_size_t
        getattr(L, n).argtypes = [cfgp]
    L.moe_forward_workspace_layout.restype = C.c_int
    L.moe_forward_workspace_layout.argtypes = [cfgp, C.POINTER(WorkspaceLayout)]
    L.moe_route.restype = C.c_int
    L.moe_route.argtypes = [cfgp, vp, vp, f32p, i32p, f32p, vp, C.c_size_t, vp]
    L.moe_permute.restype = C.c_int
    L.moe_permute.argtypes = [cfgp, vp, i32p, i32p, i32p, i32p, i32p, vp, vp, C.c_size_t, vp]
    L.moe_permute_static.restype = C.c_int
    L.moe_permute_static.argtypes = [cfgp, vp, i32p, i32p, i32p, i32p, i32p, vp, vp]
    L.moe_block_schedule.restype = C.c_int
    L.moe_block_schedule.argtypes = [cfgp, i32p, C.c_int32, i32p, i32p, vp]
    L.moe_grouped_ffn.restype = C.c_int
    L.moe_grouped_ffn.argtypes = [cfgp, vp, i32p, vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
    L.moe_pack_weights.restype = C.c_int
    L.moe_pack_weights.argtypes = [cfgp, vp, vp, vp, vp, vp]
    L.moe_combine.restype = C.c_int
    L.moe_combine.argtypes = [cfgp, vp, i32p, f32p, vp, vp]
    L.moe_forward.restype = C.c_int
    L.moe_forward.argtypes = [cfgp, vp, vp, f32p, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
    L.moe_forward_staged.restype = C.c_int
    L.moe_forward_staged.argtypes = [cfgp, vp, vp, f32p, vp, vp, vp, vp, vp, vp, C.c_size_t, vp, C.POINTER(C.c_void_p),
                                     C.c_int32]
    L.moe_test_knob.restype = C.c_int32       # test hook, not part of include/moe.h
    L.moe_test_knob.argtypes = [C.c_int32, C.c_int32]
    L.moe_test_map_launch.restype = C.c_int32  # test hook (host arithmetic only), not part of include/moe.h
    L.moe_test_map_launch.argtypes = [C.c_int32] * 5 + [i32p, i32p, C.c_int32, i32p, C.c_int32, C.c_int32, C.c_int32,
                                      C.c_int32, i32p]
    _lib = L
    return L


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors handed to the MoE library must be contiguous GPU tensors")
    return C.c_void_p(t.data_ptr())


def _stream(stream=None):
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def _check(status: int, where: str):
    if status != 0:
        raise MoEError(status, where)


def _nbytes(t) -> int:
    return t.numel() * t.element_size()


def ffn_kernel_name(cfg, stage: int, packed: bool) -> str:
    n = lib().moe_ffn_kernel_name(C.byref(cfg), stage, int(packed))
    return n.decode() if n else ""


def tile_m(cfg) -> int:
    return lib().moe_tile_m(C.byref(cfg))


def max_blocks(cfg, M: int) -> int:
    return lib().moe_max_blocks(C.byref(cfg), M)


def route_workspace_size(cfg) -> int:
    return lib().moe_route_workspace_size(C.byref(cfg))


def permute_workspace_size(cfg) -> int:
    return lib().moe_permute_workspace_size(C.byref(cfg))


def ffn_workspace_size(cfg) -> int:
    return lib().moe_ffn_workspace_size(C.byref(cfg))


def forward_workspace_size(cfg) -> int:
    return lib().moe_forward_workspace_size(C.byref(cfg))


def workspace_size(cfg) -> int:
    return lib().moe_workspace_size(C.byref(cfg))


# Test knobs of the library (csrc/moe_internal.hpp); -1 restores the selection rule.
(KNOB_GATE_UP_VARIANT, KNOB_DOWN_VARIANT, KNOB_SIDE_BY_SIDE, KNOB_EVEN_ROWS, KNOB_XCD_CHUNK, KNOB_ROT, KNOB_SHORT_NT,
 KNOB_FUSE_COMBINE, KNOB_INTERLEAVE, KNOB_NO_NT, KNOB_ROUTE_EXACT) = range(11)


def test_knob(which: int, value: int) -> int:
    """Set a test knob; returns the previous value."""
    return lib().moe_test_knob(which, value)


def map_launch(gateup: bool, ib: int, wnt: bool, N: int, M: int, offsets, blocks, blocks_mix=None, num_heavy: int = 0,
               cus: int = 256, slack_blocks: int = 0):
    """Test hook: what every workgroup of a per-block-regime GEMM launch would work on, computed on
    the host by the code the kernels run.  offsets [E+1], blocks / blocks_mix [n, 2]: numpy int32
    (host).  Returns an int32 array [grid, 6] = (has work, expert, first row, rows, feature tile,
    tile width in units of 128 features)."""
    import numpy as np
    offsets = np.ascontiguousarray(offsets, dtype=np.int32)
    blocks = np.ascontiguousarray(blocks, dtype=np.int32).reshape(-1, 2)
    nb = blocks.shape[0]
    as_p = lambda a: a.ctypes.data_as(C.POINTER(C.c_int32))
    if blocks_mix is not None:
        blocks_mix = np.ascontiguousarray(blocks_mix, dtype=np.int32).reshape(-1, 2)
        assert blocks_mix.shape[0] == nb
    max_blocks = nb + slack_blocks
    tiles = (N + 128 * ib - 1) // (128 * ib)
    capacity = (max_blocks * tiles + 7) // 8 * 8 + cus
    out = np.zeros((capacity, 6), dtype=np.int32)
    grid = lib().moe_test_map_launch(int(gateup), ib, int(wnt), N, M, as_p(offsets), as_p(blocks), nb,
                                     as_p(blocks_mix) if blocks_mix is not None else None, num_heavy, cus, max_blocks,
                                     capacity, as_p(out))
    if grid < 0:
        raise MoEError(f"moe_test_map_launch refused (gateup={gateup}, ib={ib})")
    return out[:grid]


def forward_workspace_layout(cfg) -> WorkspaceLayout:
    out = WorkspaceLayout()
    _check(lib().moe_forward_workspace_layout(C.byref(cfg), C.byref(out)), "moe_forward_workspace_layout")
    return out


def moe_route(cfg, x, W_r, bias, topk_idx, topk_w, workspace, stream=None):
    _check(lib().moe_route(C.byref(cfg), _ptr(x), _ptr(W_r), _ptr(bias), _ptr(topk_idx), _ptr(topk_w),
                           _ptr(workspace), _nbytes(workspace), _stream(stream)), "moe_route")


def moe_permute(cfg, x, topk_idx, counts, offsets, row_of, src_of, x_perm, workspace, stream=None):
    _check(lib().moe_permute(C.byref(cfg), _ptr(x), _ptr(topk_idx), _ptr(counts), _ptr(offsets), _ptr(row_of),
                             _ptr(src_of), _ptr(x_perm), _ptr(workspace), _nbytes(workspace), _stream(stream)),
           "moe_permute")


def moe_permute_static(cfg, x, topk_idx, counts, offsets, row_of, src_of, x_perm, stream=None):
    _check(lib().moe_permute_static(C.byref(cfg), _ptr(x), _ptr(topk_idx), _ptr(counts), _ptr(offsets), _ptr(row_of),
                                    _ptr(src_of), _ptr(x_perm), _stream(stream)), "moe_permute_static")


def moe_block_schedule(cfg, offsets, M, blocks, num_blocks, stream=None):
    _check(lib().moe_block_schedule(C.byref(cfg), _ptr(offsets), M, _ptr(blocks), _ptr(num_blocks),
                                    _stream(stream)), "moe_block_schedule")


def packed_weights_size(cfg) -> int:
    return lib().moe_packed_weights_size(C.byref(cfg))


def moe_pack_weights(cfg, W_gate, W_up, W_down, packed, stream=None):
    _check(lib().moe_pack_weights(C.byref(cfg), _ptr(W_gate), _ptr(W_up), _ptr(W_down), _ptr(packed),
                                  _stream(stream)), "moe_pack_weights")


def moe_grouped_ffn(cfg, x_perm, offsets, W_gate, W_up, W_down, h, y_perm, workspace, W_packed=None, stream=None):
    _check(lib().moe_grouped_ffn(C.byref(cfg), _ptr(x_perm), _ptr(offsets), _ptr(W_gate), _ptr(W_up),
                                 _ptr(W_down), _ptr(W_packed), _ptr(h), _ptr(y_perm), _ptr(workspace),
                                 _nbytes(workspace), _stream(stream)), "moe_grouped_ffn")


def moe_combine(cfg, y_perm, row_of, topk_w, y, stream=None):
    _check(lib().moe_combine(C.byref(cfg), _ptr(y_perm), _ptr(row_of), _ptr(topk_w), _ptr(y), _stream(stream)),
           "moe_combine")


def moe_forward(cfg, x, W_r, bias, W_gate, W_up, W_down, y, workspace, W_packed=None, stream=None):
    _check(lib().moe_forward(C.byref(cfg), _ptr(x), _ptr(W_r), _ptr(bias), _ptr(W_gate), _ptr(W_up),
                             _ptr(W_down), _ptr(W_packed), _ptr(y), _ptr(workspace), _nbytes(workspace),
                             _stream(stream)), "moe_forward")


def moe_forward_staged(cfg, x, W_r, bias, W_gate, W_up, W_down, y, workspace, events, W_packed=None, stream=None):
    """`events`: sequence of up to 6 hipEvent_t handles (ints) or None entries."""
    n = len(events)
    arr = (C.c_void_p * max(n, 1))(*[C.c_void_p(e) if e else None for e in events])
    _check(lib().moe_forward_staged(C.byref(cfg), _ptr(x), _ptr(W_r), _ptr(bias), _ptr(W_gate), _ptr(W_up),
                                    _ptr(W_down), _ptr(W_packed), _ptr(y), _ptr(workspace), _nbytes(workspace),
                                    _stream(stream), arr, n), "moe_forward_staged")
