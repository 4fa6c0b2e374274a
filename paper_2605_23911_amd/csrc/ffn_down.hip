// Down-projection grouped GEMM launcher: y_perm = h W_down^T  (Sec. 3.2, Eq. 4).
#include "ffn_kernels.hpp"

namespace moe {

namespace {

// See the gate+up table for the template parameters; skinny_kernel<JB, gateup, STAGES, SPLITK, packed>.
const Variant kDown[] = {
    /*0*/ {256, false, launch_tile<1, false, 3, 1, false, false>, "tile_kernel<1, false, 3, 1, false, false>"},
    /*1*/ {32, false, launch_skinny<1, false, 4, 4, false>, "skinny_kernel<1, false, 4, 4, false>"},
    /*2*/ {64, false, launch_skinny<2, false, 4, 4, false>, "skinny_kernel<2, false, 4, 4, false>"},
    /*3*/ {32, true, launch_skinny<1, false, 4, 4, true>, "skinny_kernel<1, false, 4, 4, true>"},
    /*4*/ {64, true, launch_skinny<2, false, 4, 4, true>, "skinny_kernel<2, false, 4, 4, true>"},
    /*5*/ {256, true, launch_tile_mixed<1, false, true, true>, "tile_kernel_mixed<1, false, true, true, false>"},
    /*6*/ {256, true, launch_down_mixed_wide_nt, "tile_kernel_mixed<2, false, true, true, false>"},
    /*7*/ {256, true, launch_down_mixed_wide, "tile_kernel_mixed<2, false, true, false, false>"},
    /*8*/ {128, true, launch_tile_mixed<1, false, true, true, true>, "tile_kernel_mixed<1, false, true, true, true>"},
};
constexpr int kNumDown = sizeof(kDown) / sizeof(kDown[0]);

// few_rows: the projection has too few output rows to give every CU a workgroup (T = 1 on an
// 8-expert model: 2 experts x 4096 output rows = 64 workgroups of 128 rows), so the skinny
// kernel splits K over its four wavefronts.  wide: two 32-row weight blocks per wavefront when
// that still leaves >= 512 workgroups: every token fragment read from LDS then feeds twice as
// many MFMAs and the token tile is re-read from L2 half as often per weight byte (DeepSeek-V3
// shape: 2048-long rows, 256 experts; any shape once experts hold several 256-row blocks).
int pick(int M, bool packed, const moe_config& c) {
    const long long R = (long long)c.T * c.k;
    const long long active = c.E < R ? c.E : R;
    const bool few_rows = (long long)(c.d / 128) * active < 256;
    const bool wide = (long long)(c.d / 256) * (active + R / 256) >= 512;
    if (few_rows && M <= 32) return packed ? 3 : 1;
    if (few_rows && M <= 64) return packed ? 4 : 2;
    if (!packed) return 0;   // row-major lines are consumed by four loads each: cached loads only
    if (M <= 128 && two_workgroups_per_cu(c)) return 8;
    // Per-block regime selection (tile_kernel_mixed).  Non-temporal weight loads for single-block
    // experts while the token buffers are small; with many rows per expert on average, the
    // two-weight-block form with cached loads throughout.
    const bool once = (double)R / c.E <= 192.0 && (double)R * c.d * 2.0 <= 128e6;
    if (once) return wide ? 6 : 5;
    return 7;
}

}  // namespace

bool down_fuses_combine(const moe_config& c, int32_t M, bool packed) {
    int id = forced_variant(kKnobDownVariant, kNumDown, M, packed, kDown);
    if (id < 0) id = pick(M, packed, c);
    // the per-block-regime kernels (LDS-DMA body) carry the fused epilogue; token * groups + group is an int
    return id >= 5 && (long long)c.T * combine_groups(c) < (1ll << 31);
}

const char* down_variant_name(const moe_config& c, int32_t M, bool packed) {
    int id = forced_variant(kKnobDownVariant, kNumDown, M, packed, kDown);
    if (id < 0) id = pick(M, packed, c);
    return kDown[id].name;
}

hipError_t launch_down(const moe_config& c, int32_t M, const uint16_t* h, int32_t ldh, const int32_t* offsets,
                       const int32_t* blocks, const int32_t* num_blocks, const int32_t* blocks_mix,
                       const int32_t* num_heavy, const uint16_t* wd,
                       const uint16_t* packed_dn, uint16_t* y_perm, const CombineFusion* fuse, hipStream_t s) {
    GemmArgs a{};
    a.X = h;
    a.src = nullptr;
    a.src_k = 1;
    a.x_rows = c.T * c.k;
    a.ldx = ldh;
    a.ldo = c.d;
    a.rot_mul = rot_steps(false);
    a.rot_mul_multi = rot_steps(true);
    a.W0 = wd;
    a.P = packed_dn;
    a.Out = y_perm;
    a.offsets = offsets;
    a.blocks = blocks;
    a.num_blocks = num_blocks;
    a.R = c.T * c.k;
    a.N = c.d;
    a.K = c.F;
    a.M = M;
    // token rows are addressed with 32-bit byte offsets from the buffer's base
    if ((unsigned long long)a.x_rows * (unsigned long long)ldh * 2ull >= (1ull << 32)) return hipErrorInvalidValue;
    const bool packed = packed_dn != nullptr;
    int id = forced_variant(kKnobDownVariant, kNumDown, M, packed, kDown);
    if (id < 0) id = pick(M, packed, c);
    if (kDown[id].M < M) return hipErrorInvalidValue;
    // The two-weight-block kernel with cached loads (the choice once experts hold many rows, i.e.
    // whenever routing skew has produced multi-block experts in a large batch) is also given the
    // list that holds the heavy blocks first: it deals the two classes evenly over its launch when
    // the light class is a large enough share of it, and keeps Algorithm 1's order otherwise.
    if (id == 7 && blocks_mix != nullptr && num_heavy != nullptr && knob(kKnobInterleave) != 0) {
        a.blocks_mix = blocks_mix;
        a.num_heavy = num_heavy;
        a.deal_always = knob(kKnobInterleave) > 0;
    }
    if (fuse != nullptr) {
        if (id < 5) return hipErrorInvalidValue;   // only the per-block-regime kernels have the fused epilogue
        a.comb_src = fuse->src_of;
        a.comb_row_of = fuse->row_of;
        a.comb_w = fuse->topk_w;
        a.comb_arrive = fuse->arrive;
        a.comb_y = fuse->y;
        a.comb_k = c.k;
        a.comb_groups = combine_groups(c);
    }
    return kDown[id].fn(a, moe_max_blocks(&c, M), s);
}

}  // namespace moe

// Test hook (exported, not declared in include/moe.h): enumerate on the HOST what every workgroup
// of a per-block-regime GEMM launch would work on, with the launch-order switches and the grid the
// launcher itself would use.  All array arguments are host memory.  out[w] = {has work, expert,
// first row, rows, feature tile, feature-tile width in units of 128}; returns the grid size, or -1
// if it exceeds `capacity` or (gateup, ib) names no kernel.  blocks_mix may be null (no dealing).
extern "C" __attribute__((visibility("default"))) int32_t moe_test_map_launch(
    int32_t gateup, int32_t ib, int32_t wnt, int32_t N, int32_t M, const int32_t* offsets, const int32_t* blocks,
    int32_t num_blocks, const int32_t* blocks_mix, int32_t num_heavy, int32_t cus, int32_t max_blocks, int32_t capacity,
    int32_t* out) {
    using namespace moe;
    GemmArgs a{};
    a.N = N;
    a.M = M;
    a.offsets = offsets;
    a.blocks = blocks;
    a.num_blocks = &num_blocks;
    if (blocks_mix != nullptr && knob(kKnobInterleave) != 0) {
        a.blocks_mix = blocks_mix;
        a.num_heavy = &num_heavy;
        a.deal_always = knob(kKnobInterleave) > 0;
    }
    auto run = [&](auto ibc, auto guc, auto wntc) -> int32_t {
        constexpr int IB = decltype(ibc)::value;
        constexpr bool GU = decltype(guc)::value, WNT = decltype(wntc)::value;
        const long long grid = mixed_launch_shape<IB, GU, WNT>(a, max_blocks, cus);
        if (grid > capacity) return -1;
        for (int w = 0; w < (int)grid; ++w) {
            MixedWork m{};
            const bool has = mixed_assign<IB, GU>(a, w, m);
            int32_t* o = out + 6 * (size_t)w;
            o[0] = has;
            o[1] = m.e; o[2] = m.row0; o[3] = m.rows; o[4] = m.nt;
            o[5] = m.halves ? 1 : IB;
        }
        return (int32_t)grid;
    };
    using std::integral_constant;
    using T_ = std::true_type;
    using F_ = std::false_type;
    if (gateup && ib == 1) return wnt ? run(integral_constant<int, 1>{}, T_{}, T_{}) : run(integral_constant<int, 1>{}, T_{}, F_{});
    if (!gateup && ib == 1) return wnt ? run(integral_constant<int, 1>{}, F_{}, T_{}) : run(integral_constant<int, 1>{}, F_{}, F_{});
    if (!gateup && ib == 2) return wnt ? run(integral_constant<int, 2>{}, F_{}, T_{}) : run(integral_constant<int, 2>{}, F_{}, F_{});
    return -1;
}
