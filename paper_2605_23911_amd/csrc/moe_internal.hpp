// Internal declarations shared by the library's translation units (gfx950 only).
// The public C ABI is include/moe.h; nothing here is exported.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "moe.h"

namespace moe {

constexpr int kMaxExperts = 256;      // one wavefront holds a logit row with <= 4 values per lane
constexpr int kPermChunk = 1024;      // flat slots handled by one workgroup of the permutation kernels
constexpr int kWave = 64;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// bf16 bit pattern -> float (exact).
__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// float -> bf16, round to nearest even (v_cvt_pk_bf16_f32 on gfx950).
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
    __bf16 h = (__bf16)f;
    return __builtin_bit_cast(uint16_t, h);
}

// two floats -> two bf16 in one register, lo in bits 15:0 (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi) {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// ---- test knobs -------------------------------------------------------------------------
// Process-wide integer switches that GPU tests set through moe_test_knob() (exported from the
// library, deliberately absent from include/moe.h: not part of the product interface) to force
// code paths that the selection rules would not take at test sizes.  -1 = "follow the rule".
// Nothing reads the process environment.
enum {
    kKnobGateUpVariant = 0,   // index into the gate+up variant table
    kKnobDownVariant = 1,     // index into the down-projection variant table
    kKnobSideBySide = 2,      // 0: plain tile-major order inside multi-tile experts
    kKnobEvenRows = 3,        // 0: Algorithm 1's row ranges everywhere, 3: every multi-tile expert dealt evenly
    kKnobXcdChunk = 4,        // 0/1: per-XCD contiguous chunks off/on for both projections
    kKnobRot = 5,             // k-loop rotation between the workgroups of an XCD, in steps
    kKnobShortNt = 6,         // rows up to which a multi-tile expert's last tile streams its weights non-temporally
    kKnobFuseCombine = 7,     // 0: moe_forward always launches the combine kernel, 1: folds it into the down projection whenever the kernel can
    kKnobInterleave = 8,      // 0: launch order = block order (no dealing of heavy and light blocks over the launch), 1: dealt whatever the classes' proportion
    kKnobNoNt = 9,            // 1: cached weight loads for single-block experts too
    kKnobRouteExact = 10,     // 1: every logit in fp64 at any size; 0: bf16 first pass + exact candidates from 256 tokens on
    kNumKnobs = 12
};
extern int g_knobs[kNumKnobs];
inline int knob(int i) { return g_knobs[i]; }

// ---- launchers (each enqueues on `s` and returns hipGetLastError()) ----------------------
// workspace: route_workspace_bytes(c) bytes of fp64 partial logit tiles
size_t route_workspace_bytes(const moe_config& c);
// zero / zero_per_token: if zero != nullptr the wavefront that routes token t also clears
// zero[t * zero_per_token .. + zero_per_token) (the fused combine's arrival counters).
hipError_t launch_route(const moe_config& c, const uint16_t* x, const uint16_t* wr, const float* bias,
                        int32_t* topk_idx, float* topk_w, void* workspace, int32_t* zero, int zero_per_token,
                        hipStream_t s);

// scratch: chunk histograms [nchunks, E] int32.  If blocks != nullptr the block schedule for
// tile height M is emitted by the scan kernel as well.
// blocks_mix / num_heavy (may both be null): a second list of the same blocks, as a stable
// partition into the blocks of multi-block experts and the rest, with *num_heavy (device int32) =
// size of the first class (see emit_block_schedule in permute.hip; used by the down projection).
hipError_t launch_permute_index(const moe_config& c, const int32_t* topk_idx, int32_t* counts,
                                int32_t* offsets, int32_t* row_of, int32_t* src_of, int32_t* scratch,
                                int32_t M, int32_t* blocks, int32_t* num_blocks, int32_t* blocks_mix, int32_t* num_heavy,
                                hipStream_t s);
// Device address of the current GPU's file-scope scratch array (MOE_PERMUTE_STATIC_MAX_INTS
// int32) that moe_permute_static hands to launch_permute_index in place of a caller workspace.
hipError_t permute_static_scratch(int32_t** ptr);
hipError_t launch_gather_rows(const moe_config& c, const uint16_t* x, const int32_t* src_of,
                              uint16_t* x_perm, int32_t ld_perm, hipStream_t s);
hipError_t launch_block_schedule(const moe_config& c, const int32_t* offsets, int32_t M,
                                 int32_t* blocks, int32_t* num_blocks, int32_t* blocks_mix, int32_t* num_heavy, hipStream_t s);

// packed_gu / packed_dn: the projection's region of moe_pack_weights' buffer, or nullptr to
// read the row-major weights.  gate+up reads expert-contiguous rows x_rows[R, d] when src_of is
// nullptr; otherwise x_rows is the un-permuted x[T, d] and row r is fetched from token
// src_of[r] / k (the gather of Sec. 3.1 folded into the tile load).
// ldx / ldh: row strides (elements) of x_rows and of h.
hipError_t launch_gate_up(const moe_config& c, int32_t M, const uint16_t* x_rows, int32_t ldx, const int32_t* src_of,
                          int32_t ldh, const int32_t* offsets,
                          const int32_t* blocks, const int32_t* num_blocks, const uint16_t* wg,
                          const uint16_t* wu, const uint16_t* packed_gu, uint16_t* h, hipStream_t s);
// Buffers of the weighted combine when it is folded into the down projection (Eq. 3 computed by
// the workgroup that writes the last of a token's k rows); nullptr = separate combine launch.
struct CombineFusion {
    const int32_t* src_of;   // [R]
    const int32_t* row_of;   // [T, k]
    const float* topk_w;     // [T, k]
    int32_t* arrive;         // [T, combine_groups(c)] int32, zero when the down projection starts
    uint16_t* y;             // [T, d]
};
inline int combine_groups(const moe_config& c) { return (c.d + 127) / 128; }
// whether the down-projection kernel chosen for this configuration can fold the combine in
bool down_fuses_combine(const moe_config& c, int32_t M, bool packed);
hipError_t launch_down(const moe_config& c, int32_t M, const uint16_t* h, int32_t ldh, const int32_t* offsets,
                       const int32_t* blocks, const int32_t* num_blocks, const int32_t* blocks_mix,
                       const int32_t* num_heavy, const uint16_t* wd,
                       const uint16_t* packed_dn, uint16_t* y_perm, const CombineFusion* fuse, hipStream_t s);

const char* gate_up_variant_name(const moe_config& c, int32_t M, bool packed);
const char* down_variant_name(const moe_config& c, int32_t M, bool packed);

size_t packed_gate_up_bytes(const moe_config& c);
size_t packed_down_bytes(const moe_config& c);
hipError_t launch_pack(const moe_config& c, const uint16_t* wg, const uint16_t* wu, const uint16_t* wd,
                       uint16_t* packed, hipStream_t s);

hipError_t launch_combine(const moe_config& c, const uint16_t* y_perm, const int32_t* row_of,
                          const float* topk_w, uint16_t* y, hipStream_t s);

// Many experts with a few rows each (Qwen2-MoE and DeepSeek-V3 shapes at up to 128 tokens): a
// projection is thousands of short workgroups that stream a weight panel each, and what a CU
// loses between two of them (schedule look-up, first loads, epilogue, launch of the next: ~5 us
// of ~45) shows as 10 % of the down projection.  The schedule then uses blocks of at most 128
// rows and the GEMM kernels are the builds for two workgroups per CU (half the LDS ring, at most
// 256 registers), so that one workgroup streams while its neighbour starts or ends.
// Only up to 128 tokens: no expert can then hold more than one such block, whatever the routing
// (with heavier experts under routing skew the shorter blocks and their shallower pipelines cost
// more than the overlap gains: DeepSeek-V3 shape, 512 tokens, skew 1.5: +10 %).  Only for
// launches of at least four rounds: the hardware fills a CU with two workgroups before it moves
// on, so a launch of 256 would use half the chip.
inline bool two_workgroups_per_cu(const moe_config& c) {
    const long long R = (long long)c.T * c.k;
    const long long active = c.E < R ? c.E : R;
    return c.T <= 128 && R <= 32ll * c.E && (long long)(c.d / 128) * active >= 1024;
}

inline int permute_chunks(const moe_config& c) {
    long long R = (long long)c.T * c.k;
    return (int)((R + kPermChunk - 1) / kPermChunk);
}

}  // namespace moe
