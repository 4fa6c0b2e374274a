// Fused gate+up grouped GEMM launcher: h = SiLU(x W_gate^T) (.) (x W_up^T)  (Sec. 3.3, Eq. 4).
#include "ffn_kernels.hpp"

namespace moe {

namespace {

// {tallest block, packed?, launcher, kernel template instance as rocprofv3 prints it}.
// tile_kernel<IB, gateup, STAGES, XD, packed, NT weights>,
// tile_kernel_mixed<IB, gateup, packed, NT weights for single-block experts, two workgroups per CU>.
const Variant kGateUp[] = {
    /*0*/ {256, false, launch_tile<1, true, 2, 1, false, false>, "tile_kernel<1, true, 2, 1, false, false>"},
    /*1*/ {256, true, launch_tile_mixed<1, true, true, true>, "tile_kernel_mixed<1, true, true, true, false>"},
    /*2*/ {128, true, launch_tile_mixed<1, true, true, true, true>, "tile_kernel_mixed<1, true, true, true, true>"},
};
constexpr int kNumGateUp = sizeof(kGateUp) / sizeof(kGateUp[0]);

// Packed weights: one kernel for every schedule and every routing distribution (built a second
// time for two workgroups per CU, see two_workgroups_per_cu).  It picks the
// body per block from the rows the block holds and the regime per block from the rows its expert
// holds (tile_kernel_mixed).  Row-major weights: the register-staged kernel with cached loads
// (a row-major 128-byte line is consumed by four load instructions of a lane pair, so the
// non-temporal hint would drop it between them: measured 1.7x slower).
int pick(int M, bool packed, const moe_config& c) {
    if (!packed) return 0;
    return (M <= 128 && two_workgroups_per_cu(c)) ? 2 : 1;
}

}  // namespace

const char* gate_up_variant_name(const moe_config& c, int32_t M, bool packed) {
    int id = forced_variant(kKnobGateUpVariant, kNumGateUp, M, packed, kGateUp);
    if (id < 0) id = pick(M, packed, c);
    return kGateUp[id].name;
}

hipError_t launch_gate_up(const moe_config& c, int32_t M, const uint16_t* x_rows, int32_t ldx, const int32_t* src_of,
                          int32_t ldh, const int32_t* offsets,
                          const int32_t* blocks, const int32_t* num_blocks, const uint16_t* wg,
                          const uint16_t* wu, const uint16_t* packed_gu, uint16_t* h, hipStream_t s) {
    GemmArgs a{};
    a.X = x_rows;
    a.src = src_of;
    a.src_k = c.k;
    a.x_rows = src_of ? c.T : c.T * c.k;
    a.ldx = ldx;
    a.ldo = ldh;
    a.rot_mul = rot_steps(false);
    a.rot_mul_multi = rot_steps(true);
    a.W0 = wg;
    a.W1 = wu;
    a.P = packed_gu;
    a.Out = h;
    a.offsets = offsets;
    a.blocks = blocks;
    a.num_blocks = num_blocks;
    a.R = c.T * c.k;
    a.N = c.F;
    a.K = c.d;
    a.M = M;
    // token rows are addressed with 32-bit byte offsets from the buffer's base
    if ((unsigned long long)a.x_rows * (unsigned long long)ldx * 2ull >= (1ull << 32)) return hipErrorInvalidValue;
    const bool packed = packed_gu != nullptr;
    int id = forced_variant(kKnobGateUpVariant, kNumGateUp, M, packed, kGateUp);
    if (id < 0) id = pick(M, packed, c);
    if (kGateUp[id].M < M) return hipErrorInvalidValue;
    return kGateUp[id].fn(a, moe_max_blocks(&c, M), s);
}

}  // namespace moe
