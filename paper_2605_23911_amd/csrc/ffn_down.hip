// Down-projection grouped GEMM launcher: y_perm = h W_down^T  (Sec. 3.2, Eq. 4).
#include "ffn_kernels.hpp"

namespace moe {

namespace {

const Variant kDown[] = {
    // ---- row-major weights
    /*0*/ {32, false, launch_skinny<1, false, 4, 1, false>, "skinny_kernel<1, false, 4, 1, false>"},
    /*1*/ {32, false, launch_skinny<1, false, 4, 4, false>, "skinny_kernel<1, false, 4, 4, false>"},
    /*2*/ {64, false, launch_skinny<2, false, 4, 1, false>, "skinny_kernel<2, false, 4, 1, false>"},
    /*3*/ {64, false, launch_skinny<2, false, 4, 4, false>, "skinny_kernel<2, false, 4, 4, false>"},
    /*4*/ {96, false, launch_tile<3, 1, false, 4, 2, false, false>, "tile_kernel<3, 1, false, 4, 2, false, false>"},
    /*5*/ {128, false, launch_tile<4, 1, false, 4, 2, false, false>, "tile_kernel<4, 1, false, 4, 2, false, false>"},
    /*6*/ {160, false, launch_tile<5, 1, false, 4, 2, false, false>, "tile_kernel<5, 1, false, 4, 2, false, false>"},
    /*7*/ {192, false, launch_tile<6, 1, false, 4, 2, false, false>, "tile_kernel<6, 1, false, 4, 2, false, false>"},
    /*8*/ {256, false, launch_tile<8, 1, false, 3, 1, true, false>, "tile_kernel<8, 1, false, 3, 1, true, false>"},
    // ---- packed weights
    /*9*/ {32, true, launch_skinny<1, false, 4, 1, true>, "skinny_kernel<1, false, 4, 1, true>"},
    /*10*/ {32, true, launch_skinny<1, false, 4, 4, true>, "skinny_kernel<1, false, 4, 4, true>"},
    /*11*/ {32, true, launch_tile<1, 1, false, 6, 3, false, true>, "tile_kernel<1, 1, false, 6, 3, false, true>"},
    /*12*/ {64, true, launch_skinny<2, false, 4, 4, true>, "skinny_kernel<2, false, 4, 4, true>"},
    /*13*/ {64, true, launch_tile<2, 1, false, 4, 2, false, true>, "tile_kernel<2, 1, false, 4, 2, false, true>"},
    /*14*/ {96, true, launch_tile<3, 1, false, 4, 2, false, true>, "tile_kernel<3, 1, false, 4, 2, false, true>"},
    /*15*/ {128, true, launch_tile<4, 1, false, 4, 2, false, true>, "tile_kernel<4, 1, false, 4, 2, false, true>"},
    /*16*/ {160, true, launch_tile<5, 1, false, 4, 2, false, true>, "tile_kernel<5, 1, false, 4, 2, false, true>"},
    /*17*/ {192, true, launch_tile<6, 1, false, 4, 2, false, true>, "tile_kernel<6, 1, false, 4, 2, false, true>"},
    /*18*/ {256, true, launch_tile<8, 1, false, 4, 2, true, true>, "tile_kernel<8, 1, false, 4, 2, true, true>"},
    /*19*/ {256, true, launch_tile<8, 2, false, 2, 1, true, true>, "tile_kernel<8, 2, false, 2, 1, true, true>"},
    /*20*/ {128, true, launch_tile<4, 2, false, 3, 2, false, true>, "tile_kernel<4, 2, false, 3, 2, false, true>"},
    /*21*/ {128, true, launch_tile<4, 4, false, 2, 1, false, true>, "tile_kernel<4, 4, false, 2, 1, false, true>"},
    /*22*/ {192, true, launch_tile<6, 2, false, 3, 2, false, true>, "tile_kernel<6, 2, false, 3, 2, false, true>"},
    /*23*/ {192, true, launch_tile<6, 1, false, 4, 2, false, true, 8>, "tile_kernel<6, 1, false, 4, 2, false, true, 8>"},
    /*24*/ {192, true, launch_tile<6, 2, false, 3, 2, false, true, 8>, "tile_kernel<6, 2, false, 3, 2, false, true, 8>"},
    /*25*/ {256, true, launch_tile<8, 2, false, 2, 1, true, true, 8>, "tile_kernel<8, 2, false, 2, 1, true, true, 8>"},
    /*26*/ {256, true, launch_tile<8, 2, false, 3, 2, true, true, 8>, "tile_kernel<8, 2, false, 3, 2, true, true, 8>"},
    /*27*/ {256, true, launch_tile<8, 1, false, 4, 2, true, true, 8>, "tile_kernel<8, 1, false, 4, 2, true, true, 8>"},
};
constexpr int kNumDown = sizeof(kDown) / sizeof(kDown[0]);

// few_rows: the projection has too few output rows to give every CU several workgroups, so
// the skinny kernel splits K over its four wavefronts (T = 1 on an 8-expert model: 2 experts
// x 4096 output rows = 64 workgroups otherwise).
int pick(int M, bool packed, const moe_config& c) {
    const long long R = (long long)c.T * c.k;
    const long long wgs = (long long)(c.d / 128) * (c.E < R ? c.E : R);
    const bool few_rows = wgs < 256;
    if (!packed) {
        switch (M) {
            case 32: return few_rows ? 1 : 0;
            case 64: return few_rows ? 3 : 2;
            case 96: return 4;
            case 128: return 5;
            case 160: return 6;
            case 192: return 7;
            default: return 8;
        }
    }
    switch (M) {
        case 32: return few_rows ? 10 : 11;
        case 64: return few_rows ? 12 : 13;
        case 96: return 14;
        case 128: return 15;
        case 160: return 16;
        case 192: return 17;
        default: return 18;
    }
}

}  // namespace

const char* down_variant_name(const moe_config& c, int32_t M, bool packed) {
    int id = env_variant("MOE_DN_VARIANT", kNumDown, M, packed, kDown);
    if (id < 0) id = pick(M, packed, c);
    return kDown[id].name;
}

hipError_t launch_down(const moe_config& c, int32_t M, const uint16_t* h, const int32_t* offsets,
                       const int32_t* blocks, const int32_t* num_blocks, const uint16_t* wd,
                       const uint16_t* packed_dn, uint16_t* y_perm, hipStream_t s) {
    GemmArgs a{h, wd, nullptr, packed_dn, y_perm, offsets, blocks, num_blocks, c.T * c.k, c.d, c.F, 0, 0};
    const bool packed = packed_dn != nullptr;
    int id = env_variant("MOE_DN_VARIANT", kNumDown, M, packed, kDown);
    if (id < 0) id = pick(M, packed, c);
    if (kDown[id].M != M) return hipErrorInvalidValue;
    return kDown[id].fn(a, moe_max_blocks(&c, M), s);
}

}  // namespace moe
