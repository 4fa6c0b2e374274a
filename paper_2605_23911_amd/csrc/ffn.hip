// Block-scheduled grouped GEMMs of the expert FFN on bf16 MFMA (gfx950).
// Paper: Sec. 3.2 (one launch, workgroup -> (expert, row offset) through the block schedule,
// partial tiles masked), Sec. 3.3 (gate and up projections from one shared input tile, two
// accumulators, SiLU(gate)*up in fp32 registers, a single 2-byte intermediate), Eq. 4.
//
// What differs from the paper's A100 design: the MFMA computes the TRANSPOSED tile
//     C^T[f, row] = sum_k W[f, k] * X[row, k]
// with the weight rows as the first MFMA operand.  The stored weight layout ([out, in], the
// reduction dim contiguous) is then exactly the per-lane operand layout, so weights go
// HBM -> VGPR with 16-byte loads and never touch LDS; only the (shared) token tile is staged
// in LDS.  Each of the four wavefronts owns its own weight rows and all token rows of the
// tile, so every weight byte is fetched once per workgroup.  In C^T a lane holds four
// consecutive output features of one token row, which gives 8-byte packed bf16 stores.
#include <type_traits>
#include <utility>

#include "moe_internal.hpp"

namespace moe {

namespace {

constexpr int kThreads = 256;
constexpr int kBK = 64;            // reduction elements per pipeline step
constexpr int kLdsStride = 72;     // bf16 elements per staged token row: 64 + 8 pad (144 B)

struct GemmArgs {
    const uint16_t* X;          // [R, K] expert-contiguous rows
    const uint16_t* W0;         // [E, N, K]  gate (or down)
    const uint16_t* W1;         // [E, N, K]  up   (unused for down)
    uint16_t* Out;              // [R, N]
    const int32_t* offsets;     // [E+1]
    const int32_t* blocks;      // [*, 2] (expert, row offset inside the expert)
    const int32_t* num_blocks;  // device scalar
    int R, N, K, n_tiles_n;
};

template <int... Is, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, Is...>, F&& f) {
    (f(std::integral_constant<int, Is>{}), ...);
}
// Calls f(integral_constant<0>) ... f(integral_constant<N-1>): indices are compile-time
// constants in the source, so register arrays never need a loop-unrolling pass to be promoted.
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

__device__ __forceinline__ float silu_mul(float g, float u) {
    // SiLU(g) * u with SiLU(g) = g / (1 + exp(-g)); exp(-g) = inf for very negative g gives -0.
    return g * __frcp_rn(1.0f + __expf(-g)) * u;
}

// BM: token rows per tile (Alg. 1's M).  IB: 32-row weight blocks per wavefront and matrix.
// GATEUP: two weight matrices + SwiGLU epilogue.  STAGES: weight register buffers (prefetch
// depth STAGES-1 steps).
template <int BM, int IB, bool GATEUP, int STAGES>
__global__ __launch_bounds__(kThreads) void grouped_gemm_kernel(const GemmArgs a) {
    constexpr int NM = GATEUP ? 2 : 1;
    constexpr int NI = IB * NM;          // MFMA row blocks per wavefront
    constexpr int JB = BM / 32;          // MFMA column blocks (token rows / 32)
    constexpr int BN = 4 * IB * 32;      // output features per workgroup
    constexpr int XP = BM / 32;          // 16-byte global loads per thread and step for the token tile

    __shared__ __attribute__((aligned(16))) uint16_t xs[2][BM * kLdsStride];

    const int tile = blockIdx.x / a.n_tiles_n;
    const int nt = blockIdx.x % a.n_tiles_n;
    if (tile >= *a.num_blocks) return;
    const int e = a.blocks[2 * tile];
    const int r_in = a.blocks[2 * tile + 1];
    const int seg0 = a.offsets[e];
    const int n_e = a.offsets[e + 1] - seg0;
    const int row0 = seg0 + r_in;
    const int rows = (n_e - r_in) < BM ? (n_e - r_in) : BM;

    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int li = lane & 31, half = lane >> 5;
    const int K = a.K, N = a.N;
    const int KT = K / kBK;
    const int n0w = nt * BN + wave * (IB * 32);

    // weight row pointers (row clamped so that a ragged last feature tile stays in bounds)
    const uint16_t* wp[NI];
#pragma unroll
    for (int m = 0; m < NM; ++m)
#pragma unroll
        for (int ib = 0; ib < IB; ++ib) {
            int row = n0w + ib * 32 + li;
            row = row < N ? row : N - 1;
            const uint16_t* base = (m == 0) ? a.W0 : a.W1;
            wp[m * IB + ib] = base + ((size_t)e * N + row) * K + half * 32;
        }
    // token tile: thread -> (row tid/8 + 32p, 16-byte chunk tid%8); rows clamped inside X
    const uint16_t* xp[XP];
#pragma unroll
    for (int p = 0; p < XP; ++p) {
        int row = row0 + (tid >> 3) + 32 * p;
        row = row < a.R ? row : a.R - 1;
        xp[p] = a.X + (size_t)row * K + (tid & 7) * 8;
    }
    const int xs_store = (tid >> 3) * kLdsStride + (tid & 7) * 8;
    const int xs_read = li * kLdsStride + half * 32;

    f32x16 acc[NI][JB];
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < JB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    uint4 wreg[STAGES][NI][4];
    typedef uint32_t xreg_t __attribute__((ext_vector_type(4 * XP)));
    xreg_t xreg;   // one SSA vector value (an array here is not reliably kept in registers)

    // All loads of a step are unconditional (the step index is clamped to the last one, which
    // re-reads it harmlessly) so that the loop body is straight-line code.  The token-tile loads
    // are issued BEFORE the weight prefetch of the same step: loads complete in issue order,
    // so waiting for the token tile at the end of the step leaves the newest weight loads
    // (STAGES-1 steps ahead) in flight.
    auto load_w = [&](int kt, auto st) {
        static_for<NI>([&](auto i) {
            static_for<4>([&](auto s) {
                wreg[st][i][s] = *reinterpret_cast<const uint4*>(wp[i] + (size_t)kt * kBK + s * 8);
            });
        });
    };
    auto load_x = [&](int kt) {
        static_for<XP>([&](auto p) {
            const uint4 t = *reinterpret_cast<const uint4*>(xp[p] + (size_t)kt * kBK);
            xreg[4 * p + 0] = t.x;
            xreg[4 * p + 1] = t.y;
            xreg[4 * p + 2] = t.z;
            xreg[4 * p + 3] = t.w;
        });
    };
    auto store_x = [&](int buf) {
        static_for<XP>([&](auto p) {
            *reinterpret_cast<uint4*>(&xs[buf][xs_store + p * 32 * kLdsStride]) =
                make_uint4(xreg[4 * p + 0], xreg[4 * p + 1], xreg[4 * p + 2], xreg[4 * p + 3]);
        });
    };
    auto step = [&](int kt, auto st) {
        const int buf = kt & 1;
        const int ktx = kt + 1 < KT ? kt + 1 : KT - 1;
        const int ktw = kt + STAGES - 1 < KT ? kt + STAGES - 1 : KT - 1;
        load_x(ktx);
        load_w(ktw, std::integral_constant<int, (st + STAGES - 1) % STAGES>{});
        __builtin_amdgcn_sched_barrier(0);
        static_for<4>([&](auto s) {
            bf16x8 xf[JB];
            static_for<JB>([&](auto j) {
                xf[j] = *reinterpret_cast<const bf16x8*>(&xs[buf][xs_read + j * 32 * kLdsStride + s * 8]);
            });
            static_for<NI>([&](auto i) {
                const bf16x8 wf = __builtin_bit_cast(bf16x8, wreg[st][i][s]);
                static_for<JB>([&](auto j) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xf[j], acc[i][j], 0, 0, 0);
                });
            });
        });
        __builtin_amdgcn_sched_barrier(0);
        store_x(buf ^ 1);
        __syncthreads();
    };

    // prologue: weights of the first STAGES-1 steps, token tile of step 0
    static_for<STAGES - 1>([&](auto st) { load_w(st < KT ? (int)st : KT - 1, st); });
    load_x(0);
    store_x(0);
    __syncthreads();

    int kt = 0;
    for (; kt + STAGES <= KT; kt += STAGES) static_for<STAGES>([&](auto st) { step(kt + st, st); });
    static_for<STAGES>([&](auto st) {
        if (kt + st < KT) step(kt + st, st);
    });

    // epilogue: lane holds, for token row j*32+li, features 8*(v/4) + 4*half + v%4 of each block
#pragma unroll
    for (int ib = 0; ib < IB; ++ib)
#pragma unroll
        for (int j = 0; j < JB; ++j) {
            const int tr = j * 32 + li;
            if (tr < rows) {
                uint16_t* orow = a.Out + (size_t)(row0 + tr) * N;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int f = n0w + ib * 32 + q * 8 + half * 4;
                    if (f < N) {
                        float o[4];
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            if constexpr (GATEUP)
                                o[v] = silu_mul(acc[ib][j][q * 4 + v], acc[IB + ib][j][q * 4 + v]);
                            else
                                o[v] = acc[ib][j][q * 4 + v];
                        }
                        uint2 pk;
                        pk.x = pack2_bf16(o[0], o[1]);
                        pk.y = pack2_bf16(o[2], o[3]);
                        *reinterpret_cast<uint2*>(orow + f) = pk;
                    }
                }
            }
        }
}

template <int BM, int IB, bool GATEUP, int STAGES>
hipError_t launch_variant(const GemmArgs& a, int max_blocks, hipStream_t s) {
    constexpr int BN = 4 * IB * 32;
    GemmArgs args = a;
    args.n_tiles_n = (a.N + BN - 1) / BN;
    const long long grid = (long long)max_blocks * args.n_tiles_n;
    hipLaunchKernelGGL((grouped_gemm_kernel<BM, IB, GATEUP, STAGES>), dim3((unsigned)grid), dim3(kThreads), 0, s,
                       args);
    return hipGetLastError();
}

template <bool GATEUP>
hipError_t launch_by_tile(const GemmArgs& a, int M, int max_blocks, hipStream_t s) {
    switch (M) {
        case 32:  return launch_variant<32, 1, GATEUP, 4>(a, max_blocks, s);
        case 64:  return launch_variant<64, 1, GATEUP, 3>(a, max_blocks, s);
        case 128: return launch_variant<128, 1, GATEUP, 3>(a, max_blocks, s);
        case 256: return launch_variant<256, 1, GATEUP, 2>(a, max_blocks, s);
        default:  return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_gate_up(const moe_config& c, int32_t M, const uint16_t* x_perm, const int32_t* offsets,
                          const int32_t* blocks, const int32_t* num_blocks, const uint16_t* wg,
                          const uint16_t* wu, uint16_t* h, hipStream_t s) {
    GemmArgs a{x_perm, wg, wu, h, offsets, blocks, num_blocks, c.T * c.k, c.F, c.d, 0};
    return launch_by_tile<true>(a, M, moe_max_blocks(&c, M), s);
}

hipError_t launch_down(const moe_config& c, int32_t M, const uint16_t* h, const int32_t* offsets,
                       const int32_t* blocks, const int32_t* num_blocks, const uint16_t* wd,
                       uint16_t* y_perm, hipStream_t s) {
    GemmArgs a{h, wd, nullptr, y_perm, offsets, blocks, num_blocks, c.T * c.k, c.d, c.F, 0};
    return launch_by_tile<false>(a, M, moe_max_blocks(&c, M), s);
}

}  // namespace moe
