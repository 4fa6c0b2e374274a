// Fused gate+up grouped GEMM launcher: h = SiLU(x W_gate^T) (.) (x W_up^T)  (Sec. 3.3, Eq. 4).
#include "ffn_kernels.hpp"

namespace moe {

namespace {

// {tile height, packed?, launcher}.  tile<JB, IB, gateup, STAGES, XD, DYN, packed>,
// skinny<JB, gateup, STAGES, SPLITK, packed>.
const Variant kGateUp[] = {
    // ---- row-major weights
    /*0*/ {32, false, launch_skinny<1, true, 4, 1, false>, "skinny_kernel<1, true, 4, 1, false>"},
    /*1*/ {64, false, launch_skinny<2, true, 3, 1, false>, "skinny_kernel<2, true, 3, 1, false>"},
    /*2*/ {96, false, launch_tile<3, 1, true, 3, 1, false, false>, "tile_kernel<3, 1, true, 3, 1, false, false>"},
    /*3*/ {128, false, launch_tile<4, 1, true, 3, 1, false, false>, "tile_kernel<4, 1, true, 3, 1, false, false>"},
    /*4*/ {160, false, launch_tile<5, 1, true, 3, 1, false, false>, "tile_kernel<5, 1, true, 3, 1, false, false>"},
    /*5*/ {192, false, launch_tile<6, 1, true, 3, 1, false, false>, "tile_kernel<6, 1, true, 3, 1, false, false>"},
    /*6*/ {256, false, launch_tile<8, 1, true, 2, 1, true, false>, "tile_kernel<8, 1, true, 2, 1, true, false>"},
    // ---- packed weights
    /*7*/ {32, true, launch_skinny<1, true, 4, 1, true>, "skinny_kernel<1, true, 4, 1, true>"},
    /*8*/ {32, true, launch_tile<1, 1, true, 4, 2, false, true>, "tile_kernel<1, 1, true, 4, 2, false, true>"},
    /*9*/ {64, true, launch_skinny<2, true, 3, 1, true>, "skinny_kernel<2, true, 3, 1, true>"},
    /*10*/ {64, true, launch_tile<2, 1, true, 4, 2, false, true>, "tile_kernel<2, 1, true, 4, 2, false, true>"},
    /*11*/ {96, true, launch_tile<3, 1, true, 4, 2, false, true>, "tile_kernel<3, 1, true, 4, 2, false, true>"},
    /*12*/ {128, true, launch_tile<4, 1, true, 4, 2, false, true>, "tile_kernel<4, 1, true, 4, 2, false, true>"},
    /*13*/ {160, true, launch_tile<5, 1, true, 4, 2, false, true>, "tile_kernel<5, 1, true, 4, 2, false, true>"},
    /*14*/ {192, true, launch_tile<6, 1, true, 4, 2, false, true>, "tile_kernel<6, 1, true, 4, 2, false, true>"},
    /*15*/ {256, true, launch_tile<8, 1, true, 2, 1, true, true>, "tile_kernel<8, 1, true, 2, 1, true, true>"},
    /*16*/ {128, true, launch_tile<4, 2, true, 2, 1, false, true>, "tile_kernel<4, 2, true, 2, 1, false, true>"},
    /*17*/ {160, true, launch_tile<5, 1, true, 3, 1, false, true>, "tile_kernel<5, 1, true, 3, 1, false, true>"},
    /*18*/ {32, true, launch_skinny<1, true, 6, 1, true>, "skinny_kernel<1, true, 6, 1, true>"},
    /*19*/ {192, true, launch_tile<6, 1, true, 3, 1, false, true, 8>, "tile_kernel<6, 1, true, 3, 1, false, true, 8>"},
    /*20*/ {192, true, launch_tile<6, 1, true, 2, 1, false, true, 8>, "tile_kernel<6, 1, true, 2, 1, false, true, 8>"},
    /*21*/ {192, true, launch_tile<6, 1, true, 3, 2, false, true, 8>, "tile_kernel<6, 1, true, 3, 2, false, true, 8>"},
    /*22*/ {256, true, launch_tile<8, 1, true, 2, 1, true, true, 8>, "tile_kernel<8, 1, true, 2, 1, true, true, 8>"},
    /*23*/ {256, true, launch_tile<8, 1, true, 3, 1, true, true, 8>, "tile_kernel<8, 1, true, 3, 1, true, true, 8>"},
    /*24*/ {128, true, launch_tile<4, 1, true, 4, 2, false, true, 8>, "tile_kernel<4, 1, true, 4, 2, false, true, 8>"},
};
constexpr int kNumGateUp = sizeof(kGateUp) / sizeof(kGateUp[0]);

int pick(int M, bool packed) {
    if (!packed) {
        switch (M) {
            case 32: return 0;
            case 64: return 1;
            case 96: return 2;
            case 128: return 3;
            case 160: return 4;
            case 192: return 5;
            default: return 6;
        }
    }
    switch (M) {
        case 32: return 8;
        case 64: return 10;
        case 96: return 11;
        case 128: return 12;
        case 160: return 13;
        case 192: return 14;
        default: return 15;
    }
}

}  // namespace

const char* gate_up_variant_name(const moe_config& c, int32_t M, bool packed) {
    int id = env_variant("MOE_GU_VARIANT", kNumGateUp, M, packed, kGateUp);
    if (id < 0) id = pick(M, packed);
    return kGateUp[id].name;
}

hipError_t launch_gate_up(const moe_config& c, int32_t M, const uint16_t* x_perm, const int32_t* offsets,
                          const int32_t* blocks, const int32_t* num_blocks, const uint16_t* wg,
                          const uint16_t* wu, const uint16_t* packed_gu, uint16_t* h, hipStream_t s) {
    GemmArgs a{x_perm, wg, wu, packed_gu, h, offsets, blocks, num_blocks, c.T * c.k, c.F, c.d, 0, 0};
    const bool packed = packed_gu != nullptr;
    int id = env_variant("MOE_GU_VARIANT", kNumGateUp, M, packed, kGateUp);
    if (id < 0) id = pick(M, packed);
    if (kGateUp[id].M != M) return hipErrorInvalidValue;
    return kGateUp[id].fn(a, moe_max_blocks(&c, M), s);
}

}  // namespace moe
