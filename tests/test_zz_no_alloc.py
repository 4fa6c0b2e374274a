"""moe_permute_static, the entry point that allocates nothing: its chunk histograms live in a
file-scope device array of the library instead of a caller workspace.  Checked through the C ABI
against moe_permute (bit-exact: same kernels, integer and byte results) on two calls in a row,
the second with a smaller input, so that whatever the first call left in the shared array must
not leak into the second.  Both sizes are above 8192 slots: below that the permutation runs in
one fused workgroup that needs no scratch at all."""
import os
import sys

import numpy as np
import pytest
import torch

sys.path.insert(0, os.path.dirname(__file__))

import moe_inputs as mi

pytestmark = pytest.mark.gpu


def _both(G, moe, T, E, k, alpha, seed):
    s = mi.MoEShape("static", T, 128, 64, E, k)
    idx, _ = mi.zipf_assignments(s, alpha, seed=seed)
    idx = idx.numpy()
    cfg = moe.MoEConfig.of(T, s.d, s.F, E, k)
    x = mi.make_x(s, seed).to(G.DEV)
    want = G.run_permute(cfg, idx, x)
    R = T * k
    dev_idx = torch.from_numpy(np.ascontiguousarray(idx, dtype=np.int32)).to(G.DEV)
    counts = torch.full((E,), -1, dtype=torch.int32, device=G.DEV)
    offsets = torch.full((E + 1,), -1, dtype=torch.int32, device=G.DEV)
    row_of = torch.full((R,), -1, dtype=torch.int32, device=G.DEV)
    src_of = torch.full((R,), -1, dtype=torch.int32, device=G.DEV)
    x_perm = torch.zeros((R, s.d), dtype=torch.bfloat16, device=G.DEV)
    torch.cuda.synchronize()
    moe.moe_permute_static(cfg, x, dev_idx, counts, offsets, row_of, src_of, x_perm)
    torch.cuda.synchronize()
    got = (counts.cpu().numpy(), offsets.cpu().numpy(), row_of.cpu().numpy(), src_of.cpu().numpy(), G.np_bits(x_perm))
    for name, a, b in zip(("counts", "offsets", "row_of", "src_of", "x_perm"), got, want):
        assert np.array_equal(a, b), (name, T, E, k)


def test_permute_static_equals_permute_on_two_calls_in_a_row():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2605_23911_amd as moe
    moe.lib()
    import gpu_util as G
    print("[no-alloc] first call: T=3000 E=64 k=8 (24 chunks of the shared array)", flush=True)
    _both(G, moe, 3000, 64, 8, 1.2, 5)
    print("[no-alloc] second call, smaller: T=1300 E=64 k=8 (11 chunks)", flush=True)
    _both(G, moe, 1300, 64, 8, 0.0, 6)
    # beyond the array: refused on the host, nothing enqueued
    big = moe.MoEConfig.of(40000, 128, 64, 256, 8)     # 313 chunks x 256 experts > 65536
    with pytest.raises(moe.MoEError) as err:
        t = torch.zeros(16, dtype=torch.int32, device=G.DEV)
        moe.moe_permute_static(big, None, t, t, t, t, t, None)
    assert err.value.status == -5
