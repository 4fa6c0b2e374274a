// Fused gate+up grouped GEMM launcher: h = SiLU(x W_gate^T) (.) (x W_up^T)  (Sec. 3.3, Eq. 4).
#include "ffn_kernels.hpp"

namespace moe {

namespace {

// {tallest block, packed?, launcher, kernel template instance as rocprofv3 prints it}.
// tile_kernel<IB, gateup, STAGES, XD, packed, NT weights>, tile_kernel_dma<IB, gateup, packed>,
// tile_kernel_mixed<IB, gateup, packed, NT weights for single-block experts>.
const Variant kGateUp[] = {
    /*0*/ {256, false, launch_tile<1, true, 2, 1, false, false>, "tile_kernel<1, true, 2, 1, false, false>"},
    /*1*/ {256, true, launch_tile<1, true, 2, 1, true, false>, "tile_kernel<1, true, 2, 1, true, false>"},
    /*2*/ {256, true, launch_tile<1, true, 2, 1, true, true>, "tile_kernel<1, true, 2, 1, true, true>"},
    /*3*/ {256, true, launch_tile_dma<1, true, true>, "tile_kernel_dma<1, true, true>"},
    /*4*/ {256, true, launch_tile_mixed<1, true, true, true>, "tile_kernel_mixed<1, true, true, true>"},
};
constexpr int kNumGateUp = sizeof(kGateUp) / sizeof(kGateUp[0]);

// Packed weights: one kernel for every schedule and every routing distribution.  It picks the
// body per block from the rows the block holds and the regime per block from the rows its expert
// holds (tile_kernel_mixed).  Row-major weights: the register-staged kernel with cached loads
// (a row-major 128-byte line is consumed by four load instructions of a lane pair, so the
// non-temporal hint would drop it between them: measured 1.7x slower).  Entries 1-3 are the
// register-staged kernel on packed weights and the LDS-DMA body without the per-block regime,
// for comparison runs and tests.
int pick(int M, bool packed, const moe_config& c) {
    (void)M;
    (void)c;
    return packed ? 4 : 0;
}

}  // namespace

const char* gate_up_variant_name(const moe_config& c, int32_t M, bool packed) {
    int id = env_variant("MOE_GU_VARIANT", kNumGateUp, M, packed, kGateUp);
    if (id < 0) id = pick(M, packed, c);
    return kGateUp[id].name;
}

hipError_t launch_gate_up(const moe_config& c, int32_t M, const uint16_t* x_rows, int32_t ldx, const int32_t* src_of,
                          int32_t ldh, const int32_t* offsets,
                          const int32_t* blocks, const int32_t* num_blocks, const uint16_t* wg,
                          const uint16_t* wu, const uint16_t* packed_gu, uint16_t* h, hipStream_t s) {
    GemmArgs a{x_rows, src_of, c.k, src_of ? c.T : c.T * c.k, ldx, ldh, rot_steps(false), rot_steps(true), 0, wg, wu, packed_gu, h, offsets, blocks, num_blocks, c.T * c.k, c.F, c.d, 0, M, nullptr};
    // token rows are addressed with 32-bit byte offsets from the buffer's base
    if ((unsigned long long)a.x_rows * (unsigned long long)ldx * 2ull >= (1ull << 32)) return hipErrorInvalidValue;
    const bool packed = packed_gu != nullptr;
    int id = env_variant("MOE_GU_VARIANT", kNumGateUp, M, packed, kGateUp);
    if (id < 0) id = pick(M, packed, c);
    if (kGateUp[id].M < M) return hipErrorInvalidValue;
    return kGateUp[id].fn(a, moe_max_blocks(&c, M), s);
}

}  // namespace moe
