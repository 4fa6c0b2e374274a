"""Launch order of the per-block-regime GEMM kernels, checked on the CPU.

Which workgroup computes which (rows, feature tile) of which expert is integer arithmetic on the
launch arguments and the schedule arrays (side-by-side order of an expert's row tiles, rows dealt
evenly, per-XCD chunks, a split last round, heavy and light blocks dealt over the launch).  The
library exposes that arithmetic, the very function its kernels call, through a host-side test hook;
here whole launches are enumerated for seeded random expert sizes in every order the switches
allow, and every row of every expert must be covered exactly once per 128-feature column, inside
its expert's segment, in tiles the kernel bodies can hold.  No GPU is involved."""
import itertools
import os

import numpy as np
import pytest

import paper_2605_23911_amd as moe
from paper_2605_23911_amd import binding as B
from oracle import moe_oracle as orc


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(moe.library_path()):
        from paper_2605_23911_amd import build
        build.build_library()
    return moe.lib()


@pytest.fixture
def knobs(L):
    touched = []

    def set_knob(which, value):
        touched.append(which)
        B.test_knob(which, value)
    yield set_knob
    for which in touched:
        B.test_knob(which, -1)


def _counts(rng, kind, E):
    if kind == "uniform_small":
        return rng.integers(0, 200, size=E)
    if kind == "around_tile":       # sizes near multiples of the tile heights: short last tiles, exact fits
        base = rng.choice([32, 64, 128, 256, 512, 1024], size=E)
        return np.maximum(0, base + rng.integers(-3, 40, size=E))
    if kind == "skewed":            # a few experts of thousands of rows, many small, some empty
        c = rng.integers(0, 60, size=E)
        hot = rng.choice(E, size=max(1, E // 6), replace=False)
        c[hot] = rng.integers(300, 4200, size=hot.size)
        c[rng.choice(E, size=E // 5, replace=False)] = 0
        return c
    if kind == "all_heavy":
        return rng.integers(257, 1500, size=E)
    raise ValueError(kind)


def _schedule(counts, M):
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    blocks = np.array(orc.block_schedule(offsets, M), dtype=np.int32).reshape(-1, 2)
    heavy = np.array([counts[e] > M for e, _ in blocks], dtype=bool)
    mix = np.concatenate([blocks[heavy], blocks[~heavy]]) if len(blocks) else blocks
    return offsets, blocks, mix, int(heavy.sum())


def _check_cover(work, offsets, counts, N, M, label):
    cols = (N + 127) // 128
    R = int(offsets[-1])
    cover = np.zeros((R, cols), dtype=np.int16)
    for has, e, row0, rows, nt, width in work:
        if not has:
            continue
        assert 0 <= e < len(counts), (label, e)
        assert 1 <= rows <= min(M, 256), (label, rows)
        assert offsets[e] <= row0 and row0 + rows <= offsets[e + 1], (label, e, row0, rows)
        c0 = nt * width
        # a half of a split two-block tile may lie wholly beyond a ragged N: the body then clamps its
        # weight loads into range and masks every store (it covers nothing, and must not be counted)
        assert 0 <= c0 < (cols + 1) // 2 * 2, (label, nt, width)
        cover[row0:row0 + rows, c0:min(c0 + width, cols)] += 1
    assert R == 0 or (cover.min() == 1 and cover.max() == 1), (label, int(cover.min()), int(cover.max()))


# (gate+up?, weight blocks per wavefront, non-temporal build?) of the kernels the variant tables hold
_KERNELS = [(True, 1, True), (False, 1, True), (False, 2, True), (False, 2, False)]


@pytest.mark.parametrize("kind", ["uniform_small", "around_tile", "skewed", "all_heavy"])
def test_every_row_and_feature_tile_exactly_once(L, knobs, kind):
    rng = np.random.default_rng({"uniform_small": 1, "around_tile": 2, "skewed": 3, "all_heavy": 4}[kind])
    cases = 0
    for trial in range(6):
        E = int(rng.integers(1, 40))
        counts = _counts(rng, kind, E)
        M = int(rng.choice([32, 64, 96, 128, 160, 192, 256]))
        N = int(rng.choice([64, 128, 192, 256, 640, 768, 1024, 1792, 2048, 3584]))
        offsets, blocks, mix, num_heavy = _schedule(counts, M)
        if len(blocks) == 0:
            continue
        for (gateup, ib, wnt), sib, even, chunk in itertools.product(_KERNELS, (0, 1), (0, 1, 2, 3), (0, 1)):
            knobs(B.KNOB_SIDE_BY_SIDE, sib)
            knobs(B.KNOB_EVEN_ROWS, even)
            knobs(B.KNOB_XCD_CHUNK, chunk)
            # the launcher hands the heavy-first list to the two-weight-block kernel with cached loads only
            deals = (-1, 0, 1) if (not gateup and ib == 2 and not wnt) else (0,)
            for deal in deals:
                knobs(B.KNOB_INTERLEAVE, deal)
                for cus, slack in ((256, 0), (64, 3), (8, 1)):
                    work = B.map_launch(gateup, ib, wnt, N, M, offsets, blocks, mix if deal != 0 else None, num_heavy,
                                        cus=cus, slack_blocks=slack)
                    _check_cover(work, offsets, counts, N, M,
                                 (kind, trial, E, M, N, gateup, ib, wnt, sib, even, chunk, deal, cus))
                    cases += 1
    assert cases > 500


def test_default_order_of_a_known_launch(L):
    """Hand-checked: two experts of 300 and 40 rows, M = 256, 256 features, one weight block per
    wavefront, gate+up defaults (side by side, two-tile experts dealt evenly: 160 + 140 rows)."""
    counts = np.array([300, 40])
    offsets, blocks, mix, num_heavy = _schedule(counts, 256)
    assert blocks.tolist() == [[0, 0], [0, 256], [1, 0]] and num_heavy == 2
    work = B.map_launch(True, 1, True, 256, 256, offsets, blocks)
    live = [tuple(int(v) for v in w[1:]) for w in work if w[0]]
    # expert 0: its two row tiles of feature tile 0 on one XCD class ... every (tile, feature tile) once
    assert sorted(live) == sorted([(0, 0, 160, 0, 1), (0, 0, 160, 1, 1), (0, 160, 140, 0, 1), (0, 160, 140, 1, 1),
                                   (1, 300, 40, 0, 1), (1, 300, 40, 1, 1)])
    assert len(work) == 8 and [int(w[0]) for w in work] == [1] * 6 + [0] * 2


@pytest.mark.parametrize("name,T", [("mixtral", 512), ("mixtral", 2048), ("mixtral", 4096), ("qwen2moe", 512), ("qwen2moe", 4096),
                                    ("dsv3", 512), ("dsv3", 4096), ("mixtral22", 4096)])
def test_contract_shapes_in_their_default_launch_order(L, name, T):
    """The benchmark contract's shapes at their real widths, expert sizes drawn from a multinomial
    over rank^-s popularities (s = 0, 1, 2), in the order and with the kernel forms the selection
    rules pick at that size (tile height from moe_tile_m; every kernel form is enumerated, the
    rules' choice among them)."""
    import moe_inputs as mi
    s = mi.PRESETS[name].with_T(T)
    cfg = moe.MoEConfig.of(s.T, s.d, s.F, s.E, s.k, s.gating)
    M = moe.tile_m(cfg)
    rng = np.random.default_rng(7)
    for skew in (0.0, 1.0, 2.0):
        p = np.arange(1, s.E + 1, dtype=np.float64) ** -skew
        counts = rng.multinomial(s.R, rng.permutation(p / p.sum()))
        counts = np.minimum(counts, s.T)          # an expert holds a token at most once
        offsets, blocks, mix, num_heavy = _schedule(counts, M)
        slack = moe.max_blocks(cfg, M) - len(blocks)
        assert slack >= 0
        for gateup, ib, wnt in _KERNELS:
            N = s.F if gateup else s.d
            mixed = mix if (not gateup and ib == 2 and not wnt) else None
            work = B.map_launch(gateup, ib, wnt, N, M, offsets, blocks, mixed, num_heavy, cus=256, slack_blocks=slack)
            _check_cover(work, offsets, counts, N, M, (name, T, skew, gateup, ib, wnt))
