// Block-scheduled grouped GEMMs of the expert FFN on bf16 MFMA (gfx950).
// Paper: Sec. 3.2 (one launch, workgroup -> (expert, row offset) through the block schedule,
// partial tiles masked), Sec. 3.3 (gate and up projections from one shared input tile, two
// accumulators, SiLU(gate)*up in fp32 registers, a single 2-byte intermediate), Eq. 4.
//
// What differs from the paper's A100 design: the MFMA computes the TRANSPOSED tile
//     C^T[f, row] = sum_k W[f, k] * X[row, k]
// with the weight rows as the first MFMA operand.  The stored weight layout ([out, in], the
// reduction dim contiguous) is then exactly the per-lane operand layout, so weights go
// HBM -> VGPR with 16-byte loads and never touch LDS.  The MFMA sums over k, so which k a
// fragment slot carries is free as long as both operands agree: MFMA s of a 64-wide step takes
// k = 16 s + 8 (lane / 32) + 0..7, which makes the two lanes of a weight row read 32 contiguous
// bytes per load instruction (one 64-byte L1 access instead of two).  Each wavefront owns its own weight rows
// and all token rows of the tile, so every weight byte is fetched once per workgroup.  In C^T
// a lane holds four consecutive output features of one token row (8-byte packed bf16 stores).
//
// PACKED weights: lanes of one load instruction read 32 different weight rows, 16 bytes each,
// which costs one L1 access per lane.  moe_pack_weights re-orders the weights once (weights are
// static at inference) into the order the loads consume them, [expert][32-row block][64-k step]
// [matrix][s][lane] x 16 bytes, so that one load instruction reads 1 KiB contiguous and a
// wavefront streams one contiguous region.  Both layouts are supported by every kernel.
//
// Kernels that share that mapping:
//   tile_kernel        token tile (up to 256 rows) staged in LDS through registers and shared by
//                      the four wavefronts; body chosen per block from the rows it holds.
//   tile_kernel_mixed  the same tile brought global -> LDS by DMA into a ring of buffers, with
//                      the regime chosen per block: weights streamed
//                      once (non-temporal, k rotated) for experts that fit one block, shared
//                      through L2 (cached, k in step, row tiles side by side) for experts that
//                      span several (the default for packed weights).
//   skinny_kernel      <= 64 token rows, token fragments loaded straight from L2 by each
//                      wavefront: no LDS, no barrier in the reduction loop; the four wavefronts
//                      split K (down projection of few-expert models at a handful of tokens,
//                      where there are too few output rows to fill 256 CUs otherwise).
#pragma once

#include <type_traits>
#include <utility>

#include "moe_internal.hpp"

namespace moe {

struct GemmArgs {
    const uint16_t* X;          // [R, K] expert-contiguous rows, or the un-permuted [T, K] rows if src != nullptr
    const int32_t* src;         // [R] flat (token, slot) index of every expert-contiguous row, or nullptr
    int src_k;                  // slots per token: row r then lives at X[src[r] / src_k]
    int x_rows;                 // rows of X (T with a source map, else R); x_rows * ldx * 2 bytes < 4 GiB
    int ldx, ldo;               // row strides of X and Out in elements (>= K and >= N)
    int rot_mul;                // k-loop rotation between workgroups of one XCD, in steps (see tile_body)
    int rot_mul_multi;          // the same for blocks of experts that span several row tiles (tile_kernel_mixed)
    int slots;                  // workgroups the chip runs at once (one per CU); 0 = do not split the last round
    const uint16_t* W0;         // [E, N, K]  gate (or down)
    const uint16_t* W1;         // [E, N, K]  up   (unused for down)
    const uint16_t* P;          // packed weights of this projection (PACKED kernels), else unused
    uint16_t* Out;              // [R, N]
    const int32_t* offsets;     // [E+1]
    const int32_t* blocks;      // [*, 2] (expert, row offset inside the expert)
    const int32_t* num_blocks;  // device scalar
    const int32_t* num_heavy;   // device scalar or null: the first *num_heavy blocks belong to multi-block experts (tile_kernel_mixed)
    int R, N, K, n_tiles_n;
    int M;                      // tile height of the block schedule (rows per block <= M)
    int sib;                    // tile_kernel_mixed: launch the row tiles of one expert side by side (see there)
    int chunk;                  // tile_kernel_mixed: one contiguous eighth of the work per XCD (see there)
    const int32_t* blocks_mix;  // with num_heavy: the same blocks, those of multi-block experts first (the list the dealt order reads)
    int deal_always;            // tile_kernel_mixed with num_heavy: deal the two classes whatever their proportion (tests)
    int even;                   // tile_kernel_mixed: rows of a multi-tile expert dealt evenly over its schedule entries
    int no_nt;                  // tile_kernel_mixed: cached weight loads for every block (test knob)
    int short_nt;               // tile_kernel_mixed: tiles of at most this many rows stream their weights non-temporally
    // Weighted combine folded into the down projection (all null / 0 when it is a separate launch):
    const int32_t* comb_src;    // [R] flat (token, slot) index of every expert-contiguous row
    const int32_t* comb_row_of; // [T, k] expert-contiguous row of every (token, slot)
    const float* comb_w;        // [T, k] gate weights
    int32_t* comb_arrive;       // [T, comb_groups] rows of the token written so far per 128-feature group (zero at launch)
    uint16_t* comb_y;           // [T, N] layer output
    int comb_k, comb_groups;    // experts per token; ceil(N / 128)
};

typedef hipError_t (*launch_fn)(const GemmArgs&, int, hipStream_t);

// The down projection's per-block-regime kernels with two weight blocks per wavefront are
// compiled in a translation unit of their own (ffn_down_wide.hip) to shorten the build.
hipError_t launch_down_mixed_wide_nt(const GemmArgs& a, int max_blocks, hipStream_t s);
hipError_t launch_down_mixed_wide(const GemmArgs& a, int max_blocks, hipStream_t s);

namespace {

constexpr int kThreads = 256;
constexpr int kBK = 64;            // reduction elements per pipeline step
constexpr int kLdsStride = 72;     // bf16 elements per staged token row: 64 + 8 pad (144 B)


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

// Weight loads.  NT: when an expert is a single block each PACKED weight byte is used exactly
// once per launch (one load instruction consumes whole 128-byte lines), and loading it with the
// non-temporal hint keeps the streamed weights from evicting the re-used token tiles from L2
// (+5..10 % at T <= 512).  When an expert spans several row blocks they share the weight panel
// through L2 and the hint would defeat that; so it would for row-major weights, where a line is
// consumed by four load instructions.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
template <bool NT>
__device__ __forceinline__ uint4 load_w16(const uint16_t* p) {
    if constexpr (NT) {
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
        return make_uint4(v[0], v[1], v[2], v[3]);
    } else {
        return *reinterpret_cast<const uint4*>(p);
    }
}

__device__ __forceinline__ float silu_mul(float g, float u) {
    // SiLU(g) * u with SiLU(g) = g / (1 + exp(-g)); exp(-g) = inf for very negative g gives -0.
    // v_rcp_f32 (1 ulp) on purpose: the correctly rounded reciprocal expands to a ten-instruction
    // division, which made up 40 % of the epilogue; the result is rounded to bf16 right after.
    return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u;
}

// Buffer addressing (buffer_load_dwordx4 ... offen): address = descriptor base (scalar) + scalar
// offset + per-lane 32-bit offset + immediate.  The per-step advance along k is the scalar offset
// and the per-lane offset never changes, so the loads of the reduction loop need no vector
// address arithmetic and no 64-bit address registers.  Offsets beyond the descriptor's range
// read as zero instead of faulting.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);   // raw, 32-bit data format
}
template <bool NT>
__device__ __forceinline__ uint4 buffer_load16(rsrc_t r, uint32_t lane_off, uint32_t scalar_off) {
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, lane_off, scalar_off, NT ? 2 : 0);
    return make_uint4(v[0], v[1], v[2], v[3]);
}

// Weight fragment addressing.  Unpacked: row-major rows, element (row, k).  Packed: 16-byte
// units ordered [expert][row block][k step][matrix][s][lane].
template <bool PACKED, int NM>
struct WAddr {
    static constexpr int kStep = PACKED ? NM * 4 * 512 : kBK;   // elements per 64-wide k step
    static constexpr int sStep = PACKED ? 512 : 16;              // elements per MFMA slot s
    // A fragment address is block() + lane_bytes(): block() is the same for the whole wavefront
    // (it lives in scalar registers and the per-step advance is scalar arithmetic), lane_bytes()
    // is a 32-bit per-lane offset that never changes, so a load needs no per-step vector
    // address arithmetic and no 64-bit address registers.
    __device__ static __forceinline__ int clamp_block(const GemmArgs& a, int row_block) {
        const int last = PACKED ? a.N / 32 - 1 : (a.N - 1) / 32;   // ragged last feature tile: stores are masked
        return row_block < last ? row_block : last;
    }
    __device__ static __forceinline__ const uint16_t* block(const GemmArgs& a, int e, int row_block, int m) {
        const int rb = clamp_block(a, row_block);
        if constexpr (PACKED)
            return a.P + ((size_t)e * (a.N / 32) + rb) * (size_t)(a.K / kBK) * kStep + m * 4 * 512;
        else
            return (m == 0 ? a.W0 : a.W1) + ((size_t)e * a.N + rb * 32) * a.K;
    }
    // bytes from block() to the end of the rows / packed region it belongs to (buffer range)
    __device__ static __forceinline__ uint32_t block_bytes(const GemmArgs& a, int row_block, int m) {
        if constexpr (PACKED) {
            return (uint32_t)(a.K / kBK) * kStep * 2u - (uint32_t)m * 4096u;
        } else {
            const int rows = a.N - clamp_block(a, row_block) * 32;
            return (uint32_t)(rows < 32 ? rows : 32) * (uint32_t)a.K * 2u;
        }
    }
    __device__ static __forceinline__ uint32_t lane_bytes(const GemmArgs& a, int row_block, int lane) {
        if constexpr (PACKED) {
            return (uint32_t)lane * 16u;
        } else {
            const int li = lane & 31, half = lane >> 5;
            const int rb = clamp_block(a, row_block);
            int row = rb * 32 + li;
            row = (row < a.N ? row : a.N - 1) - rb * 32;
            return (uint32_t)(row * a.K + half * 8) * 2u;
        }
    }
    __device__ static __forceinline__ const uint16_t* base(const GemmArgs& a, int e, int row_block, int m, int lane) {
        return block(a, e, row_block, m) + lane_bytes(a, row_block, lane) / 2;
    }
};

// Address of expert-contiguous token row `row` (clamped to the last row).  With a source map the
// permutation of Sec. 3.1 is applied here, in the load address, and the permuted copy of the
// activations is never written.
__device__ __forceinline__ int token_row_index(const GemmArgs& a, int row) {
    row = row < a.R ? row : a.R - 1;
    if (a.src != nullptr) row = a.src[row] / a.src_k;
    return row;
}
__device__ __forceinline__ const uint16_t* token_row(const GemmArgs& a, int row) {
    return a.X + (size_t)token_row_index(a, row) * a.ldx;
}
// Byte offset of a token row from a.X as 32 bits (the launchers refuse buffers of 4 GiB or more).
__device__ __forceinline__ uint32_t token_row_bytes(const GemmArgs& a, int row) {
    return (uint32_t)token_row_index(a, row) * (uint32_t)a.ldx * 2u;
}

// Block schedule entry -> tile geometry (Alg. 1: block = (expert, row offset)).
struct Tile {
    int e, row0, rows;
    int n_e;   // rows of the whole expert
};
__device__ __forceinline__ bool load_tile(const GemmArgs& a, int tile, int BM, Tile& t) {
    BM = a.M < BM ? a.M : BM;   // a kernel may serve a schedule with shorter blocks than it can hold
    if (tile >= *a.num_blocks) return false;
    t.e = a.blocks[2 * tile];
    const int r_in = a.blocks[2 * tile + 1];
    const int seg0 = a.offsets[t.e];
    const int n_e = a.offsets[t.e + 1] - seg0;
    t.row0 = seg0 + r_in;
    t.rows = (n_e - r_in) < BM ? (n_e - r_in) : BM;
    t.n_e = n_e;
    return true;
}

// Workgroup -> (tile, feature tile): tile-major, feature tiles of one block-schedule entry
// adjacent.  The hardware deals workgroups to the 8 XCDs round-robin; with a feature-tile count
// that is a multiple of 8 the row tiles of one expert that share a weight panel land on the
// same XCD (and run at about the same time), so the panel is fetched into one L2 only.
// (Measured: cutting the work into 8 contiguous per-XCD chunks instead is slower at large T
// because it separates exactly those row tiles in time.)
__device__ __forceinline__ bool map_workgroup(const GemmArgs& a, int& tile, int& nt) {
    tile = blockIdx.x / a.n_tiles_n;
    nt = blockIdx.x - tile * a.n_tiles_n;
    return true;
}

// Epilogue for one 32x32 MFMA block: the lane holds, for token row (j*32 + lane%32), the
// features q*8 + 4*(lane/32) + 0..3 (q = 0..3) of the block that starts at feature f0.  The two
// lanes of a row (lane and lane^32) swap halves so that each writes two 16-byte pieces (lane/32
// = 0: features 0..7 and 16..23, lane/32 = 1: 8..15 and 24..31) instead of four 8-byte ones:
// half as many store instructions and write requests.  Every lane of the wavefront must call
// this (the swap is a cross-lane operation); `live` masks the stores of rows beyond the tile.
// DEVICE_SCOPE: the 16-byte pieces are written with device-scope (sc1) stores, which go through
// to the level all XCDs share, so that a workgroup on another XCD can read them after this
// wavefront has waited for its stores and bumped a counter (fused combine), without an L2
// write-back.
template <bool GATEUP, bool DEVICE_SCOPE = false>
__device__ __forceinline__ void store_block(const f32x16& g, const f32x16& u, uint16_t* out_row, int f0, int half,
                                            int N, bool live) {
    uint2 pk[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        float o[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) o[v] = GATEUP ? silu_mul(g[q * 4 + v], u[q * 4 + v]) : g[q * 4 + v];
        pk[q].x = pack2_bf16(o[0], o[1]);
        pk[q].y = pack2_bf16(o[2], o[3]);
    }
#pragma unroll
    for (int p = 0; p < 2; ++p) {   // pair p: groups q = 2p (kept by half 0) and q = 2p + 1 (kept by half 1)
        const uint2 give = half ? pk[2 * p] : pk[2 * p + 1];
        uint2 got;
        got.x = __shfl_xor(give.x, 32, kWave);
        got.y = __shfl_xor(give.y, 32, kWave);
        const int f = f0 + (2 * p + half) * 8;
        const uint4 v = half ? make_uint4(got.x, got.y, pk[2 * p + 1].x, pk[2 * p + 1].y)
                             : make_uint4(pk[2 * p].x, pk[2 * p].y, got.x, got.y);
        if (live && f < N) {
            if constexpr (DEVICE_SCOPE) {
                // one-row descriptor: base = the row, range = N elements
                const u32x4 d4 = {v.x, v.y, v.z, v.w};
                __builtin_amdgcn_raw_buffer_store_b128(d4, make_rsrc(out_row, (uint32_t)N * 2u), (uint32_t)f * 2u, 0, 16);
            } else {
                *reinterpret_cast<uint4*>(out_row + f) = v;
            }
        }
    }
}

// =============================================================================================
// tile_body: up to 256 token rows (JBE blocks of 32) staged in LDS through registers and shared
// by the four wavefronts; each wavefront owns IB 32-row weight blocks per matrix and ALL token
// rows of the tile.
// =============================================================================================
template <int JBE, int IB, bool GATEUP, int STAGES, int XD, bool PACKED, bool WNT>
__device__ __forceinline__ void tile_body(const GemmArgs& a, const Tile& t, int nt, uint16_t* xs) {
    constexpr int NM = GATEUP ? 2 : 1;
    constexpr int NI = IB * NM;
    constexpr int BM = 256;                     // rows one LDS buffer is laid out for
    constexpr int BN = 4 * IB * 32;
    constexpr int JW = JBE;                     // 32-row token blocks per wavefront
    constexpr int XROWS = kThreads / 8;         // token rows staged per pass (8 threads x 16 B per row)
    constexpr int XP = (JBE * 32) / XROWS;      // passes per step
    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);   // wave-uniform: scalar register
    const int li = lane & 31, half = lane >> 5;
    const int K = a.K, N = a.N;
    const int KT = K / kBK;
    const int n0w = nt * BN + wave * (IB * 32);

    // Weight fragments: scalar block base per (matrix, row block) + one per-lane byte offset.
    // Out-of-range rows of a ragged last feature tile are clamped, their stores masked.
    typedef WAddr<PACKED, NM> WA;
    rsrc_t wb[NI];
    uint32_t wl[PACKED ? 1 : IB];
    static_for<NM>([&](auto m) {
        static_for<IB>([&](auto ib) {
            wb[m * IB + ib] = make_rsrc(WA::block(a, t.e, n0w / 32 + ib, m), WA::block_bytes(a, n0w / 32 + ib, m));
        });
    });
    static_for<(PACKED ? 1 : IB)>([&](auto ib) { wl[ib] = WA::lane_bytes(a, n0w / 32 + ib, lane); });
    auto w_load = [&](auto i, int kc, auto s) {
        return buffer_load16<WNT>(wb[i], wl[PACKED ? 0 : i % IB] + s * (WA::sStep * 2), (uint32_t)kc * (WA::kStep * 2));
    };
    const rsrc_t xb = make_rsrc(a.X, (uint32_t)a.x_rows * (uint32_t)a.ldx * 2u);
    // token tile: thread -> (row tid/8 + XROWS*p, 16-byte chunk tid%8); rows clamped inside X.
    // Scalar base a.X + k offset, per-thread 32-bit byte offsets fixed for the whole loop.
    uint32_t xo[XP];
    static_for<XP>([&](auto p) {
        xo[p] = token_row_bytes(a, t.row0 + (tid >> 3) + XROWS * p) + (uint32_t)(tid & 7) * 16u;
    });
    const int xs_store = (tid >> 3) * kLdsStride + (tid & 7) * 8;
    const int xs_read = li * kLdsStride + half * 8;

    f32x16 acc[NI][JW];
    static_for<NI>([&](auto i) {
        static_for<JW>([&](auto j) {
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
        });
    });

    uint4 wreg[STAGES][NI][4];
    typedef uint32_t xreg_t __attribute__((ext_vector_type(4 * XP)));
    xreg_t xreg[XD];   // each set is one SSA vector value (a plain array is not reliably kept in registers)

    // The K loop is rotated per workgroup: logical step i reads physical step (i + rot) mod KT.
    // All rows of a token tile at one k step are a whole multiple of 4 KiB apart when the row
    // length is (d = 4096, F = 14336, ...), so they sit in the same L2 channel; workgroups that
    // run together on an XCD (ids 8 apart) start two steps apart and so spread over the channels
    // instead of all hammering the same one.  The sum over k does not care about the order.
    const int rot = (int)(((blockIdx.x >> 3) * (unsigned)a.rot_mul) % (unsigned)KT);
    auto phys = [&](int i) {
        int p = (i < KT ? i : KT - 1) + rot;
        return p >= KT ? p - KT : p;
    };

    // Software pipeline.  In step kt the wavefront issues the token-tile loads of step kt+XD and
    // the weight loads of step kt+STAGES-1, runs the MFMAs of step kt from LDS buffer kt%2 and
    // its weight registers, then writes the token tile of step kt+1 (loaded XD-1 steps ago) into
    // the other LDS buffer.  Loads complete in issue order, so that last wait leaves everything
    // issued later in flight.  All loads are unconditional (the step index is clamped to the
    // last step, which is re-read harmlessly): straight-line code.
    auto load_w = [&](int kt, auto st) {
        const int kc = phys(kt);
        static_for<NI>([&](auto i) {
            static_for<4>([&](auto s) {
                wreg[st][i][s] = w_load(i, kc, s);
            });
        });
    };
    auto load_x = [&](int kt, auto xs_) {
        const uint32_t kb = (uint32_t)phys(kt) * (kBK * 2);
        static_for<XP>([&](auto p) {
            const uint4 v = buffer_load16<false>(xb, xo[p], kb);
            xreg[xs_][4 * p + 0] = v.x;
            xreg[xs_][4 * p + 1] = v.y;
            xreg[xs_][4 * p + 2] = v.z;
            xreg[xs_][4 * p + 3] = v.w;
        });
    };
    auto store_x = [&](int buf, auto xs_) {
        static_for<XP>([&](auto p) {
            *reinterpret_cast<uint4*>(&xs[buf * BM * kLdsStride + xs_store + p * XROWS * kLdsStride]) =
                make_uint4(xreg[xs_][4 * p + 0], xreg[xs_][4 * p + 1], xreg[xs_][4 * p + 2], xreg[xs_][4 * p + 3]);
        });
    };
    // One step.  Whatever a wavefront does between MFMAs leaves the matrix pipe idle unless it
    // is issued while an MFMA is still executing (or another wavefront of the SIMD has MFMAs
    // ready).  The weight loads of the prefetched step and the LDS fragment reads of the next
    // slot are therefore spread between the MFMA groups (one group = one weight fragment against
    // all token blocks); sched_barrier pins that order, which the compiler's scheduler would undo.
    // `u` = kt modulo the unroll factor UNR (a multiple of both STAGES and XD), compile-time.
    auto step = [&](int kt, auto u) {
        const int buf = kt & 1;
        constexpr int wst = (u + STAGES - 1) % STAGES;
        const int kw = phys(kt + STAGES - 1);
        load_x(kt + XD, std::integral_constant<int, (u + XD) % XD>{});           // set (kt+XD)%XD == kt%XD
        bf16x8 xf[2][JW];
        static_for<JW>([&](auto j) {
            xf[0][j] = *reinterpret_cast<const bf16x8*>(&xs[buf * BM * kLdsStride + xs_read + j * 32 * kLdsStride]);
        });
        __builtin_amdgcn_sched_barrier(0);
        static_for<4>([&](auto s) {
            static_for<NI>([&](auto i) {
                const bf16x8 wf = __builtin_bit_cast(bf16x8, wreg[u % STAGES][i][s]);
                static_for<JW>([&](auto j) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xf[s & 1][j], acc[i][j], 0, 0, 0);
                    constexpr int p = i * JW + j;   // position in the slot: one memory instruction behind each MFMA
                    if constexpr (j == 0) wreg[wst][i][s] = w_load(i, kw, s);
                    if constexpr (s < 3 && p % NI == NI - 1) {
                        constexpr int jj = p / NI;
                        xf[(s + 1) & 1][jj] = *reinterpret_cast<const bf16x8*>(
                            &xs[buf * BM * kLdsStride + xs_read + jj * 32 * kLdsStride + (s + 1) * 16]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                });
            });
        });
        store_x(buf ^ 1, std::integral_constant<int, (u + 1) % XD>{});            // token tile of step kt+1
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
    };
    // NOTE on register sets: in step kt the set kt%XD is free (its tile, step kt, went to LDS at
    // the end of step kt-1), so the loads of step kt+XD reuse it; with XD == 1 the single set is
    // loaded at the top of the step and stored at its end.

    static_for<STAGES - 1>([&](auto st) { load_w(st, st); });
    load_x(0, std::integral_constant<int, 0>{});
    store_x(0, std::integral_constant<int, 0>{});
    static_for<XD - 1>([&](auto q) { load_x(q + 1, std::integral_constant<int, (q + 1) % XD>{}); });
    __syncthreads();

    constexpr int UNR = (STAGES % XD == 0) ? STAGES : STAGES * XD;
    int kt = 0;
    for (; kt + UNR <= KT; kt += UNR) static_for<UNR>([&](auto u) { step(kt + u, u); });
    static_for<UNR>([&](auto u) {
        if (kt + u < KT) step(kt + u, u);
    });

    static_for<IB>([&](auto ib) {
        static_for<JW>([&](auto j) {
            const int tr = j * 32 + li;
            const bool live = tr < t.rows;
            store_block<GATEUP>(acc[ib][j], acc[GATEUP ? IB + ib : ib][j],
                                a.Out + (size_t)(t.row0 + (live ? tr : 0)) * a.ldo, n0w + ib * 32, half, N, live);
        });
    });
}

// ---------------------------------------------------------------------------------------------
// tile_body_dma: same tile, but the token tile goes global -> LDS with the gfx950 LDS-DMA load
// (global_load_lds_dwordx4: each lane supplies its own global address, the 64 x 16 bytes land
// contiguously at M0 + 16*lane), so it needs no staging registers, no ds_write, and can be
// prefetched XD steps ahead into a ring of XD+1 LDS buffers.  LDS rows are 128 bytes, unpadded
// (the DMA fixes the destination order); bank conflicts are avoided by permuting the SOURCE:
// position p of row r holds chunk p ^ swz(r), swz(r) = (r ^ (r >> 3)) & 7, and the fragment
// reads apply the same XOR.  The DMA is issued from inline assembly so that the compiler does
// not serialise every later LDS read behind it; completion is awaited with an explicit
// s_waitcnt vmcnt(N) before the step's barrier (loads complete in issue order; N = the number
// of vector-memory loads this wavefront issues after the batch it waits for).  Memory operations
// the compiler adds on its own (a spill) cannot break the wait: while the awaited DMA is
// outstanding the N later loads are outstanding too, so the counter is above N; extra operations
// only lengthen the wait.
// ---------------------------------------------------------------------------------------------
// M0 is on the clobber list so that the compiler never orders this statement between its own
// write of M0 and the instruction that consumes it.  M0 is a reserved (non-allocatable)
// register, for which clang prints a generic "may not be preserved" warning: overwriting it is
// exactly what is declared here, so the warning is silenced for this one statement.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void lds_dma16(const void* gptr, uint32_t lds_addr) {
    const uint32_t base = __builtin_amdgcn_readfirstlane(lds_addr);   // wave-uniform: goes through M0
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(base)
                 : "memory", "m0");
}
#pragma clang diagnostic pop
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
    // gfx9 encoding: vmcnt[3:0] -> bits 3:0, vmcnt[5:4] -> bits 15:14; expcnt (6:4) and lgkmcnt (11:8) = no wait
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// Weighted combine (Eq. 3) folded into the down projection: the paper's limitation 1, second
// half.  The k rows of a token come from k different experts, i.e. from workgroups that run at
// different times on different XCDs, each with an L2 of its own.  A device-scope fence pair
// (write back and invalidate the whole L2 around every tile) measured 1.4-2.7x on the down
// projection; instead the tile of y_perm is written with device-scope stores, the wavefronts wait
// for their acknowledgement, and the rows are read back with device-scope loads.  Each workgroup,
// once its tile is written, adds 1 to a counter per (token, 128-feature group) for every row it
// holds (device-scope atomics); whoever brings a counter to k knows that all k rows of that token and group are in
// memory, reads them back and forms
//     y[t, c] = sum_i w[t, i] * y_perm[row_of[t, i], c]
// in fp32 in slot order i = 0..k-1 from the bf16 values in memory, its own row included: the
// same arithmetic on the same operands as the stand-alone combine kernel, whichever workgroup
// arrives last, so y is bit-reproducible and bit-equal to moe_combine's.  No workgroup ever waits
// for another.  The counters are cleared by the router (the wavefront that routes token t clears
// token t's counters), so no extra launch and no host-side reset is involved.
// `nt` is the index of the workgroup's feature tile of width 128 * IB; xs is LDS that the
// reduction loop no longer uses.
template <int IB>
__device__ __forceinline__ void fused_combine(const GemmArgs& a, const Tile& t, int nt, uint16_t* xs) {
    int* list_n = reinterpret_cast<int*>(xs);
    int* list = list_n + 4;            // up to rows * IB entries: token * groups + group
    const int tid = threadIdx.x;
    const int groups = a.comb_groups, k = a.comb_k;
    wait_vmcnt<0>();                   // this wavefront's device-scope y_perm stores have been acknowledged
    __syncthreads();                   // ... and so have the other wavefronts'; LDS is free (all LDS-DMAs have landed too)
    if (tid == 0) *list_n = 0;
    __syncthreads();
    for (int r = tid; r < t.rows; r += kThreads) {
        const int token = a.comb_src[t.row0 + r] / k;
#pragma unroll
        for (int ib = 0; ib < IB; ++ib) {
            const int g = nt * IB + ib;
            if (g < groups) {
                const int old = atomicAdd(&a.comb_arrive[(size_t)token * groups + g], 1);
                if (old == k - 1) list[atomicAdd(list_n, 1)] = token * groups + g;
            }
        }
    }
    __syncthreads();
    const int n = *list_n;
    if (n == 0) return;
    const int sub = tid & 15;          // 16 lanes x 16 bytes = one 128-feature group of one row
    const uint32_t row_bytes = (uint32_t)a.ldo * 2u;
    const rsrc_t out_rows = make_rsrc(a.Out, (uint32_t)a.R * row_bytes);   // < 4 GiB: checked by the launcher
    for (int q = tid >> 4; q < n; q += kThreads / 16) {
        const int tg = list[q];
        const int token = tg / groups, g = tg - token * groups;
        const int c = g * 128 + sub * 8;
        if (c >= a.N) continue;
        const int32_t* rows = a.comb_row_of + (size_t)token * k;
        const float* w = a.comb_w + (size_t)token * k;
        float acc[8];
#pragma unroll
        for (int v = 0; v < 8; ++v) acc[v] = 0.0f;
        // Eight rows are requested before the first is used (the workgroup has its CU to itself:
        // nothing else hides the latency of these loads); the sum still runs in slot order.
        for (int i0 = 0; i0 < k; i0 += 8) {
            u32x4 v[8];
            float wi[8];
#pragma unroll
            for (int b = 0; b < 8; ++b) {
                const int i = i0 + b < k ? i0 + b : k - 1;
                // device-scope (sc1) load: served from the level all XCDs share, never from a line this XCD cached earlier
                v[b] = __builtin_amdgcn_raw_buffer_load_b128(out_rows, (uint32_t)rows[i] * row_bytes + (uint32_t)c * 2u, 0, 16);
                wi[b] = w[i];
            }
#pragma unroll
            for (int b = 0; b < 8; ++b) {
                if (i0 + b < k) {
#pragma unroll
                    for (int p = 0; p < 4; ++p) {
                        acc[2 * p] = fmaf(wi[b], __uint_as_float(v[b][p] << 16), acc[2 * p]);
                        acc[2 * p + 1] = fmaf(wi[b], __uint_as_float(v[b][p] & 0xffff0000u), acc[2 * p + 1]);
                    }
                }
            }
        }
        uint4 o;
        o.x = pack2_bf16(acc[0], acc[1]);
        o.y = pack2_bf16(acc[2], acc[3]);
        o.z = pack2_bf16(acc[4], acc[5]);
        o.w = pack2_bf16(acc[6], acc[7]);
        *reinterpret_cast<uint4*>(a.comb_y + (size_t)token * a.N + c) = o;
    }
}

template <int JB, int JBE, int IB, bool GATEUP, int STAGES, int XD, bool PACKED, bool WNT = false>
__device__ __forceinline__ void tile_body_dma(const GemmArgs& a, const Tile& t, int nt, uint16_t* xs) {
    constexpr int NM = GATEUP ? 2 : 1;
    constexpr int NI = IB * NM;
    constexpr int BN = 4 * IB * 32;
    constexpr int NBUF = XD + 1;
    constexpr int BUF_BYTES = JBE * 32 * 128;
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int li = lane & 31, half = lane >> 5;
    const int K = a.K, N = a.N;
    const int KT = K / kBK;
    const int n0w = nt * BN + wave * (IB * 32);

    typedef WAddr<PACKED, NM> WA;
    const uint16_t* wp[NI];
    static_for<NM>([&](auto m) {
        static_for<IB>([&](auto ib) { wp[m * IB + ib] = WA::base(a, t.e, n0w / 32 + ib, m, lane); });
    });
    // DMA q of this wavefront covers the 8 rows rg*8.., rg = 4q + wave: lane -> row rg*8 + lane/8,
    // LDS position lane%8, source chunk position ^ swz(row) with swz = ((lane>>3) ^ rg) & 7.
    const uint16_t* xp[JBE];
    static_for<JBE>([&](auto q) {
        const int rg = q * 4 + wave;
        const int chunk = (lane & 7) ^ (((lane >> 3) ^ rg) & 7);
        xp[q] = token_row(a, t.row0 + rg * 8 + (lane >> 3)) + chunk * 8;
    });
    const uint32_t lds0 = (uint32_t)(uintptr_t)xs;            // LDS byte address of the ring
    const uint32_t dma_dst = lds0 + wave * 1024;              // + q*4096 + buffer*BUF_BYTES
    // fragment reads: row j*32 + li, logical chunk 2s + half, swizzle (li ^ li>>3 ^ 4(j&1)) & 7
    const int sw0 = (li ^ (li >> 3)) & 7;
    int rd_off[2][4];   // [j parity][slot] byte offset inside a row
    static_for<2>([&](auto pj) {
        static_for<4>([&](auto s) { rd_off[pj][s] = (((2 * s + half) ^ (sw0 ^ (pj * 4))) & 7) * 16; });
    });
    const char* xs_b = reinterpret_cast<const char*>(xs) + li * 128;

    f32x16 acc[NI][JBE];
    static_for<NI>([&](auto i) {
        static_for<JBE>([&](auto j) {
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
        });
    });
    uint4 wreg[STAGES][NI][4];

    const int rot = (int)(((blockIdx.x >> 3) * (unsigned)a.rot_mul) % (unsigned)KT);   // see tile_body
    auto phys = [&](int i) {
        int p = (i < KT ? i : KT - 1) + rot;
        return p >= KT ? p - KT : p;
    };
    auto load_w = [&](int kt, auto st) {
        const int kc = phys(kt);
        static_for<NI>([&](auto i) {
            static_for<4>([&](auto s) {
                wreg[st][i][s] = load_w16<WNT>(wp[i] + (size_t)kc * WA::kStep + s * WA::sStep);
            });
        });
    };
    auto dma_x = [&](int kt, int buf) {
        const int kc = phys(kt);
        static_for<JBE>([&](auto q) { lds_dma16(xp[q] + (size_t)kc * kBK, dma_dst + buf * BUF_BYTES + q * 4096); });
    };
    auto frag = [&](int buf, auto j, auto s) {
        return *reinterpret_cast<const bf16x8*>(xs_b + buf * BUF_BYTES + j * 4096 + rd_off[j & 1][s]);
    };
    // The token tile of step kt+2 (not kt+1) is awaited at the end of step kt, so a tile is
    // visible to every wavefront one whole step before it is used; the first fragments of step
    // kt+1 can then be read during the last slot of step kt and the MFMAs of the next step
    // start right behind the barrier instead of behind an LDS round trip.
    // The DMA instructions of a step are dealt over its MFMA groups (group g takes q = g, g+NG,
    // ...) behind that group's weight load: the CU's one address unit needs 16 cycles per
    // 64-lane 16-byte access, and a burst of JBE of them from all four wavefronts at once would
    // hold every instruction stream (and so the MFMAs) for several hundred cycles per step.
    // Loads this wavefront issues after its last DMA of step kt+2-XD and before the end of step
    // kt: the weight loads of the groups behind that DMA, then (XD-2) whole steps.
    static_assert(XD >= 2, "needs the tile of step kt+2 in flight during step kt");
    constexpr int NG = 4 * NI;                                   // MFMA groups = weight loads per step
    constexpr int G_LAST = (JBE < NG ? JBE : NG) - 1;            // last group that issues a DMA
    constexpr int VM_AFTER = (NG - 1 - G_LAST) + (XD - 2) * (NG + JBE);

    bf16x8 xnext[JBE];   // slot-0 fragments of the next step
    // One wavefront per SIMD: while it issues a run of memory instructions nothing feeds the
    // matrix pipe, which holds one MFMA (32 cycles) ahead at most.  So the memory instructions
    // of a slot (per group one weight load and the group's share of the token-tile DMAs, JBE
    // fragment reads for the next slot) are dealt singly between its NI*JBE MFMAs: fragment jj of the next slot
    // behind MFMA jj*NI + NI-1, i.e. still NI*JBE - jj*(NI-1) - NI + 1 >= JBE MFMAs before its
    // use.  (Issuing them as one run at the head of each group measured 5 % slower.)
    auto step = [&](int kt, auto u) {
        const int buf = kt % NBUF;
        constexpr int wst = (u + STAGES - 1) % STAGES;
        const int kw = phys(kt + STAGES - 1);
        const int kx = phys(kt + XD);
        const uint32_t dst = dma_dst + ((kt + XD) % NBUF) * BUF_BYTES;   // the buffer read in step kt-1: free since that step's barrier
        bf16x8 xf[2][JBE];
        static_for<JBE>([&](auto j) { xf[0][j] = xnext[j]; });
        __builtin_amdgcn_sched_barrier(0);
        static_for<4>([&](auto s) {
            static_for<NI>([&](auto i) {
                const bf16x8 wf = __builtin_bit_cast(bf16x8, wreg[u % STAGES][i][s]);
                static_for<JBE>([&](auto j) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xf[s & 1][j], acc[i][j], 0, 0, 0);
                    constexpr int p = i * JBE + j;               // position of this MFMA in the slot
                    constexpr int jd = JBE > 2 ? 2 : JBE - 1;    // the group's DMA goes behind this MFMA
                    if constexpr (j == 0)
                        wreg[wst][i][s] = load_w16<WNT>(wp[i] + (size_t)kw * WA::kStep + s * WA::sStep);
                    if constexpr (j == jd) {
                        static_for<JBE>([&](auto q) {
                            if constexpr (q % NG == s * NI + i) lds_dma16(xp[q] + (size_t)kx * kBK, dst + q * 4096);
                        });
                    }
                    if constexpr (p % NI == NI - 1) {
                        constexpr int jj = p / NI;
                        if constexpr (s < 3)
                            xf[(s + 1) & 1][jj] = frag(buf, std::integral_constant<int, jj>{}, std::integral_constant<int, (s + 1) % 4>{});
                        else   // last slot: slot-0 fragments of the next step (its tile is visible since the previous barrier)
                            xnext[jj] = frag((kt + 1) % NBUF, std::integral_constant<int, jj>{}, std::integral_constant<int, 0>{});
                    }
                    __builtin_amdgcn_sched_barrier(0);
                });
            });
        });
        wait_vmcnt<VM_AFTER>();   // this wavefront's share of the token tile of step kt+2 has landed
        __syncthreads();
    };

    // prologue: token tiles of steps 0..XD-1, weights of steps 0..STAGES-2; tiles 0 and 1 complete
    static_for<XD>([&](auto q) { dma_x(q, q % NBUF); });
    static_for<STAGES - 1>([&](auto st) { load_w(st, st); });
    wait_vmcnt<(XD - 2) * JBE + (STAGES - 1) * NI * 4>();
    __syncthreads();
    static_for<JBE>([&](auto j) { xnext[j] = frag(0, j, std::integral_constant<int, 0>{}); });

    constexpr int UNR = STAGES;
    int kt = 0;
    for (; kt + UNR <= KT; kt += UNR) static_for<UNR>([&](auto u) { step(kt + u, u); });
    static_for<UNR>([&](auto u) {
        if (kt + u < KT) step(kt + u, u);
    });
    wait_vmcnt<0>();   // nothing of this workgroup may still be writing LDS when it retires

    if constexpr (!GATEUP) {
        if (a.comb_arrive != nullptr) {
            static_for<IB>([&](auto ib) {
                static_for<JBE>([&](auto j) {
                    const int tr = j * 32 + li;
                    const bool live = tr < t.rows;
                    store_block<GATEUP, true>(acc[ib][j], acc[ib][j], a.Out + (size_t)(t.row0 + (live ? tr : 0)) * a.ldo,
                                              n0w + ib * 32, half, N, live);
                });
            });
            return fused_combine<IB>(a, t, nt, xs);
        }
    }
    static_for<IB>([&](auto ib) {
        static_for<JBE>([&](auto j) {
            const int tr = j * 32 + li;
            const bool live = tr < t.rows;
            store_block<GATEUP>(acc[ib][j], acc[GATEUP ? IB + ib : ib][j],
                                a.Out + (size_t)(t.row0 + (live ? tr : 0)) * a.ldo, n0w + ib * 32, half, N, live);
        });
    });
}

// DYN (256-row tiles only): the body is chosen per tile from the rows it really holds, so one
// launch serves experts of any size: a 20-row expert runs the 32-row body, a 1000-row expert
// four 256-row tiles.  This is the "dynamic block-to-expert assignment" the paper leaves as
// future work (its Sec. 4.7 and limitation 5): Algorithm 1 runs with M = 256 and the tile
// height inside a block follows n_e.  Empty token blocks cost neither loads, LDS traffic nor
// MFMA issue slots.  Pipeline depths per body are what the register file allows.
// Body of the 256-row dynamic-height kernel for a block of t.rows rows (four wavefronts).
template <int IB, bool GATEUP, int STAGES, int XD, bool PACKED, bool WNT>
__device__ __forceinline__ void tile_dispatch(const GemmArgs& a, const Tile& t, int nt, uint16_t* xs) {
    constexpr int NI = IB * (GATEUP ? 2 : 1);
    constexpr int SD = NI >= 4 ? 3 : 4;          // stages for the small bodies
    constexpr int S56 = NI >= 4 ? 2 : SD;
    switch ((t.rows + 31) / 32) {
        case 1: return tile_body<1, IB, GATEUP, SD, 2, PACKED, WNT>(a, t, nt, xs);
        case 2: return tile_body<2, IB, GATEUP, SD, 2, PACKED, WNT>(a, t, nt, xs);
        case 3: return tile_body<3, IB, GATEUP, SD, 2, PACKED, WNT>(a, t, nt, xs);
        case 4: return tile_body<4, IB, GATEUP, SD, 2, PACKED, WNT>(a, t, nt, xs);
        case 5: return tile_body<5, IB, GATEUP, S56, 2, PACKED, WNT>(a, t, nt, xs);
        case 6: return tile_body<6, IB, GATEUP, S56, 2, PACKED, WNT>(a, t, nt, xs);
        default: return tile_body<8, IB, GATEUP, STAGES, XD, PACKED, WNT>(a, t, nt, xs);
    }
}

template <int IB, bool GATEUP, int STAGES, int XD, bool PACKED, bool WNT>
__global__ __launch_bounds__(kThreads) void tile_kernel(const GemmArgs a) {
    extern __shared__ __attribute__((aligned(16))) uint16_t xs[];
    Tile t;
    int tile, nt;
    if (!map_workgroup(a, tile, nt) || !load_tile(a, tile, 256, t)) return;
    tile_dispatch<IB, GATEUP, STAGES, XD, PACKED, WNT>(a, t, nt, xs);
}

// The dynamic-height kernel with the LDS-DMA token tile.  LDS: (XD+1) buffers of up to 32 KiB.
template <int IB, bool GATEUP, bool PACKED, bool WNT = false, bool HALF = false>
__device__ __forceinline__ void dma_dispatch(const GemmArgs& a, const Tile& t, int nt, uint16_t* xs) {
    constexpr int NI = IB * (GATEUP ? 2 : 1);
    constexpr int SD = NI >= 4 ? 3 : 4;
    if constexpr (HALF) {   // blocks of at most 128 rows, two workgroups per CU: register budget 256 per wavefront
        switch ((t.rows + 31) / 32) {
            case 1: return tile_body_dma<8, 1, IB, GATEUP, 3, 3, PACKED, WNT>(a, t, nt, xs);
            case 2: return tile_body_dma<8, 2, IB, GATEUP, 3, 3, PACKED, WNT>(a, t, nt, xs);
            case 3: return tile_body_dma<8, 3, IB, GATEUP, 2, 3, PACKED, WNT>(a, t, nt, xs);
            default: return tile_body_dma<8, 4, IB, GATEUP, 2, 3, PACKED, WNT>(a, t, nt, xs);
        }
    }
    switch ((t.rows + 31) / 32) {
        case 1: return tile_body_dma<8, 1, IB, GATEUP, SD, 3, PACKED, WNT>(a, t, nt, xs);
        case 2: return tile_body_dma<8, 2, IB, GATEUP, SD, 3, PACKED, WNT>(a, t, nt, xs);
        case 3: return tile_body_dma<8, 3, IB, GATEUP, SD, 3, PACKED, WNT>(a, t, nt, xs);
        case 4: return tile_body_dma<8, 4, IB, GATEUP, SD, 3, PACKED, WNT>(a, t, nt, xs);
        case 5: return tile_body_dma<8, 5, IB, GATEUP, NI >= 4 ? 2 : SD, 3, PACKED, WNT>(a, t, nt, xs);
        case 6: return tile_body_dma<8, 6, IB, GATEUP, NI >= 4 ? 2 : SD, 3, PACKED, WNT>(a, t, nt, xs);
        case 7: return tile_body_dma<8, 7, IB, GATEUP, 3, 3, PACKED, WNT>(a, t, nt, xs);
        default: return tile_body_dma<8, 8, IB, GATEUP, 3, 3, PACKED, WNT>(a, t, nt, xs);
    }
}

// The regime is a property of the EXPERT, not of the launch: under routing skew a few experts
// hold thousands of rows while most hold a handful.  This kernel decides per block; both regimes
// run the LDS-DMA body.  An expert that fits one block streams its weights once: non-temporal
// weight loads if WNT, k loop rotated against its XCD neighbours.  An expert that spans several
// row tiles shares its weight panels through L2: cached weight loads, k walked in step, its row
// tiles launched side by side.  (Packed weights.  The register-staged body of tile_kernel was the
// single-block choice until the memory instructions of the DMA body were dealt singly between
// its MFMAs; since then the DMA body wins there too: no staging registers, no ds_write, half the
// instructions per token-tile byte.  Mixtral shape: T=512 layer -3 %, T=1024 -5 %, T <= 256 and
// the 64- and 256-expert shapes unchanged.)
//
// Last round (IB = 2 only).  The grid runs in rounds of `slots` workgroups, one per CU.  With
// two weight blocks per wavefront a projection has few, heavy workgroups (Mixtral shape, down
// projection at T=2048: 320 = 1.25 rounds); when the last round is at most half full, each of
// its workgroups is replaced by two that take one 128-feature half each with the IB = 1 body,
// so the round lasts about half as long and uses twice the CUs.  Only when at most one full
// round precedes it: with many rounds the workgroups do not end together, there is no common
// "last round" to shorten, and the less efficient halves cost more than they gain (measured:
// -10 % at T=2048, +3..5 % at T=4096 and T=8192 without this condition).
//
// mixed_assign: what workgroup w of a tile_kernel_mixed launch works on.  Integer arithmetic on the launch
// arguments and the schedule arrays only, callable on the host as well: the CPU tests enumerate
// whole launches with it (host copies of the arrays) and check that every (row, feature tile) of
// every expert is covered exactly once in each launch order.
struct MixedWork {
    int e, row0, rows, n_e;   // expert, first expert-contiguous row, rows of this workgroup, rows of the expert
    int nt;                   // feature tile: of IB * 128 features, or of 128 when `halves`
    bool halves;              // IB == 2 down projection: one 128-feature half of a tile of the split last round (IB = 1 body)
};
template <int IB, bool GATEUP>
__host__ __device__ inline bool mixed_assign(const GemmArgs& a, const int wg, MixedWork& m) {
    int tile, nt;
    bool halves = false, chunked = false, dealt = false;
    const int32_t* blist = a.blocks;   // Algorithm 1's order unless the two classes are dealt (below)
    const int total = *a.num_blocks * a.n_tiles_n;
    int split_from = total;            // first position (in two-block tiles) of a split last round
    {
        int w = wg, sub = 0;
        bool split_round = false;
        if constexpr (IB == 2 && !GATEUP) {
            if (a.slots > 0) {
                const int full = total / a.slots * a.slots, rem = total - full;
                split_round = rem > 0 && 2 * rem <= a.slots && full <= a.slots;
                if (split_round) split_from = full;
                if (split_round && w >= full) {
                    const int h = w - full;
                    w = full + (h >> 1);
                    sub = h & 1;
                    halves = true;
                }
            }
        }
        // One contiguous eighth of the (tile-major) work per XCD: the hardware deals workgroup id
        // to XCD id % 8, so XCD x takes ids x*per .. x*per+per-1.  All feature tiles of a block
        // then run on one XCD and its token tile is fetched into one L2 instead of eight (down
        // projection, single-block experts: the h tile of an expert is read by d/128 workgroups
        // and makes up half of what a CU loads).
        if (a.chunk && !split_round) {
            const int per = (total + 7) >> 3;
            const int q = w >> 3;
            if (q >= per) return false;
            w = (w & 7) * per + q;
            chunked = true;
        }
        if (w >= total) return false;
        // Heavy and light blocks dealt evenly over the launch.  With a.num_heavy the block list
        // holds the blocks of multi-block experts first (their workgroups are bound by the matrix
        // cores and leave HBM mostly alone), then the single-block experts (bound by the weight
        // stream).  Launched in that order, or in expert order under routing skew, the chip runs
        // stretches of one kind only: all CUs compute while HBM idles, then all CUs stream and
        // share the bandwidth.  Position p of the launch therefore takes the next unit of the
        // class that a proportional (Bresenham) merge puts there, so that at any time the resident
        // workgroups are a mix in the launch's own proportion: the streaming ones then have the
        // memory system to themselves.  The unit is 8 consecutive ids where the feature-tile count
        // is a multiple of 8 (id % 8, the XCD, and the side-by-side order below are kept), else
        // one block.  Both classes keep their ascending expert order, so the light experts' weights
        // are still read in address order.  Uniform routing has one class only: nothing moves.
        // Dealing costs the heavy class: row tiles that share a weight panel no longer start
        // together (a few percent of their time, whatever the light class holds), and what it
        // gains grows with the light class's share of the launch.  It is therefore done only
        // when the single-block experts number at least 2/5 of the multi-block experts' blocks
        // (measured at T=4096: DeepSeek-V3 shape, 173 / 65 / 31 light against ~130 heavy blocks:
        // -9.6 %, -5.6 %, -1.8 %; Qwen2-MoE shape, 40 / 45 / 32 against ~130: +2.6 %, +2.8 %, +5.5 %).
        if (a.num_heavy != nullptr && !chunked && !split_round) {
            const int U = (a.n_tiles_n & 7) == 0 ? 8 : a.n_tiles_n;
            const int hb = *a.num_heavy, lb = *a.num_blocks - hb;
            const int hu = hb * a.n_tiles_n / U, tu = total / U, lu = tu - hu;
            if (hu > 0 && lu > 0 && (a.deal_always || 5 * lb >= 2 * hb)) {
                blist = a.blocks_mix;
                const int p = w / U, r = w - p * U;
                // heavy units among positions [0, p): floor(p * hu / tu); position p is heavy iff that count steps at p
                const long long before = (long long)p * hu / tu, upto = (long long)(p + 1) * hu / tu;
                const int unit = upto > before ? (int)before : hu + (p - (int)before);
                w = unit * U + r;
                dealt = U != 8;   // whole units of 8 ids keep an expert's workgroups on the XCDs the order below assumes
            }
        }
        tile = w / a.n_tiles_n;
        nt = w - tile * a.n_tiles_n;
        if (halves) nt = 2 * nt + sub;   // index of the 128-feature tile the IB = 1 body works on
    }
    // Row tiles of one expert side by side.  The workgroups of an expert with n row tiles are a
    // contiguous span of n * n_tiles_n launch positions; the hardware deals workgroup id to XCD
    // id % 8, so the positions of the span that are 8 apart (one "class", position % 8) run on one
    // XCD, one after the other.  In plain tile-major order the n workgroups that read the same
    // weight panel are n_tiles_n positions apart: they start microseconds apart, on whatever XCD
    // that distance leads to, and an XCD's 4 MiB of L2 hold only about three k steps of its 32
    // workgroups' streams, so each of them fetches the panel from beyond L2 for itself.  Inside
    // the span the order is therefore (feature tile, row tile) per class: the n row tiles of a
    // panel are consecutive positions of one class, i.e. consecutive workgroups of one XCD, start
    // together and walk k in step.  A class of c positions holds c / n whole panels; the c % n
    // positions left over in each class take the remaining panels' tiles in turn (those panels are
    // spread over several XCDs; none when n_tiles_n is a multiple of 8).  A short last tile (a
    // different, faster body) would not stay in step anyway: those go to the end of the span.
    // (Mixtral shape, T=4096: layer -3 %; T=8192 -2 %; no effect on single-tile experts.)
    // The schedule entry is read once: the look-ups (block count, entry, expert offsets, for
    // the gate+up projection the source row) are dependent loads in front of the block's first
    // weight and tile loads, each worth several hundred nanoseconds of a ~100 us block.
    if (tile >= *a.num_blocks) return false;
    const int bm = a.M < 256 ? a.M : 256;              // rows per schedule entry
    const int e = blist[2 * tile];
    const int r_in = blist[2 * tile + 1];
    const int seg0 = a.offsets[e];
    const int n_e = a.offsets[e + 1] - seg0;
    const int n = (n_e + bm - 1) / bm;                 // row tiles (schedule entries) of this expert
    int ti = r_in / bm;                                // which of them this workgroup is
    // see below; a.even: 0 never, 1 experts of up to three row tiles, 2 those while the launch is at most two rounds, 3 always
    const bool even = a.even == 3 || (n <= 3 && (a.even == 1 || (a.even == 2 && total <= 2 * a.slots)));
    // An expert whose span reaches into a split last round keeps the plain order in all of its
    // workgroups, the halves and the whole tiles before them alike: the two orders number the
    // positions of a span differently, so one span must use one of them throughout.
    const bool in_split = (tile - ti + n) * a.n_tiles_n > split_from;
    if (a.sib && !in_split && !chunked && !dealt && n >= 2) {
        auto body = [](int rows) { const int c = (rows + 31) >> 5; return c > 7 ? 8 : c; };
        // tiles that run the same body as the first one (all of them when the rows are dealt evenly)
        const int nf = (even || body(n_e - (n - 1) * bm) == body(bm)) ? n : n - 1;
        const int l = ti * a.n_tiles_n + nt;           // position inside the expert's span
        const int span = nf * a.n_tiles_n;             // positions of the tiles that keep pace with each other
        if (l >= span) {
            ti = n - 1;
            nt = l - span;
        } else {
            const int cls = l & 7, j = l >> 3;         // class of the position, index inside the class
            int left_before = 0, whole = 0, mine = 0;
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const int positions = (span - c + 7) >> 3, panels = positions / nf;   // non-increasing in c
                if (c < cls) left_before += positions - panels * nf;
                if (c == cls) mine = panels;
                whole += panels;
            }
            if (j < mine * nf) {
                // the p-th whole panel of every class: panels p * 8 + class (at any time the XCDs work on neighbouring panels)
                nt = (j / nf) * 8 + cls;
                ti = j % nf;
            } else {
                const int m = left_before + (j - mine * nf);
                nt = whole + m / nf;
                ti = m % nf;
            }
        }
    }
    // Rows of a multi-tile expert dealt evenly over its n schedule entries, in whole 32-row blocks:
    // Algorithm 1 gives 1040 rows as 4 x 256 + 16, and the 16-row tile streams a whole weight
    // panel for 1/16 of the MFMA work, eight times faster through k than its siblings, so it
    // shares nothing with them (1040 instead of 1024 rows per expert cost +8 % on gate+up and
    // +15 % on the down projection).  5 x 224 (4 x 224 + 144) is the same number of 32-row MFMA
    // blocks, ceil(n_e / 32), in tiles that run at about the same pace.  Which rows a workgroup
    // computes does not change any row's result.  The CU time of the two divisions is about the
    // same (a 16-row tile costs a third of a full one); what differs is how the launch ends.
    // Experts of two or three row tiles, where the short tile's extra pass over the weight panel
    // is a third to a half of the expert's weight traffic, are dealt evenly (Mixtral shape T=1024
    // -4 %, T=2048 -5 %, Qwen2-MoE shape T=4096 -2 %); with four tiles or more the 224-row bodies
    // cost what the shared panel saves (gate+up at T=4096 +1.7 %).  Down projection (few, heavy
    // workgroups): only while the launch is at most two rounds, where equal tiles end together
    // (T=2048: 538 -> 455 us); with more rounds the quick short tiles fill the gaps better
    // (T=4096: 864 against 915 us).
    int row_in = ti * bm, rows = bm;
    if (even && n >= 2) {
        const int per = (((n_e + n - 1) / n) + 31) & ~31;   // <= 256
        row_in = ti * per;
        rows = per;
    }
    rows = (n_e - row_in) < rows ? (n_e - row_in) : rows;
    if (rows <= 0) return false;                            // (n >= 8 only: the rounding can empty the last entry)
    m.e = e;
    m.row0 = seg0 + row_in;
    m.rows = rows;
    m.n_e = n_e;
    m.nt = nt;
    m.halves = halves;
    return true;
}

// The kernel: what to work on from mixed_assign, the regime from the expert's rows, the body from the block's.
template <int IB, bool GATEUP, bool PACKED, bool WNT, bool HALF = false>
__global__ __launch_bounds__(kThreads, HALF ? 2 : 1) void tile_kernel_mixed(const GemmArgs a) {
    extern __shared__ __attribute__((aligned(1024))) uint16_t xs[];
    MixedWork m;
    if (!mixed_assign<IB, GATEUP>(a, (int)blockIdx.x, m)) return;
    Tile t;
    const int nt = m.nt;
    const bool halves = m.halves;
    t.e = m.e;
    t.row0 = m.row0;
    t.rows = m.rows;
    t.n_e = m.n_e;
    GemmArgs b = a;
    // A short last tile of a multi-tile expert runs through k several times faster than its
    // siblings and shares nothing with them in time: it streams the panel like a single-block
    // expert does (non-temporal, k rotated), so that its stream does not evict the panels the
    // full tiles share.
    const bool multi = t.n_e > a.M && t.rows > a.short_nt;
    if (multi) b.rot_mul = a.rot_mul_multi;
    const bool shared = multi || a.no_nt;
    if constexpr (IB == 2 && !GATEUP) {
        if (halves) {
            if (shared) return dma_dispatch<1, GATEUP, PACKED, false, HALF>(b, t, nt, xs);
            return dma_dispatch<1, GATEUP, PACKED, WNT, HALF>(b, t, nt, xs);
        }
    }
    if (shared) return dma_dispatch<IB, GATEUP, PACKED, false, HALF>(b, t, nt, xs);
    dma_dispatch<IB, GATEUP, PACKED, WNT, HALF>(b, t, nt, xs);
}

// =============================================================================================
// skinny_kernel: JB*32 <= 64 token rows, fragments straight from global memory, no LDS in the
// reduction loop.  SPLITK == 1: the four wavefronts own four different 32-row weight blocks.
// SPLITK == 4: they share one weight block and each reduces a quarter of K; partial sums are
// added in wavefront order through LDS (fixed order: bit-reproducible).
// =============================================================================================
template <int JB, bool GATEUP, int STAGES, int SPLITK, bool PACKED, bool WNT = true>
__global__ __launch_bounds__(kThreads) void skinny_kernel(const GemmArgs a) {
    constexpr int NM = GATEUP ? 2 : 1;
    constexpr int BM = JB * 32;
    constexpr int BN = (SPLITK == 1) ? 128 : 32;
    __shared__ float red[(SPLITK == 1) ? 1 : 3 * NM * JB * 16 * kWave];

    Tile t;
    int tile, nt;
    if (!map_workgroup(a, tile, nt) || !load_tile(a, tile, BM, t)) return;
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int li = lane & 31, half = lane >> 5;
    const int K = a.K, N = a.N;
    const int KT = K / kBK;
    const int n0w = nt * BN + (SPLITK == 1 ? wave * 32 : 0);
    const int per = (KT + SPLITK - 1) / SPLITK;
    const int kt_begin = (SPLITK == 1) ? 0 : wave * per;
    // last step of this wavefront's K range; below kt_begin when the range is empty
    const int kt_last = ((SPLITK == 1) ? KT : ((kt_begin + per) < KT ? (kt_begin + per) : KT)) - 1;

    typedef WAddr<PACKED, NM> WA;
    const uint16_t* wp[NM];
    static_for<NM>([&](auto m) { wp[m] = WA::base(a, t.e, n0w / 32, m, lane); });
    const uint16_t* xp[JB];
    static_for<JB>([&](auto j) {
        xp[j] = token_row(a, t.row0 + j * 32 + li) + half * 8;
    });

    f32x16 acc[NM][JB];
    static_for<NM>([&](auto i) {
        static_for<JB>([&](auto j) {
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
        });
    });

    uint4 wreg[STAGES][NM][4];
    uint4 xreg[STAGES][JB][4];
    auto load = [&](int kt, auto st) {
        int kc = kt < kt_last ? kt : kt_last;   // clamped into [0, KT): always in bounds
        kc = kc > 0 ? kc : 0;
        static_for<NM>([&](auto i) {
            static_for<4>([&](auto s) {
                wreg[st][i][s] = load_w16<WNT>(wp[i] + (size_t)kc * WA::kStep + s * WA::sStep);
            });
        });
        static_for<JB>([&](auto j) {
            static_for<4>([&](auto s) {
                xreg[st][j][s] = *reinterpret_cast<const uint4*>(xp[j] + (size_t)kc * kBK + s * 16);
            });
        });
    };
    auto step = [&](int kt, auto st) {
        load(kt + STAGES - 1, std::integral_constant<int, (st + STAGES - 1) % STAGES>{});
        __builtin_amdgcn_sched_barrier(0);
        static_for<4>([&](auto s) {
            static_for<NM>([&](auto i) {
                static_for<JB>([&](auto j) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8, wreg[st][i][s]), __builtin_bit_cast(bf16x8, xreg[st][j][s]),
                        acc[i][j], 0, 0, 0);
                });
            });
        });
        __builtin_amdgcn_sched_barrier(0);
    };

    static_for<STAGES - 1>([&](auto st) { load(kt_begin + st, st); });
    int kt = kt_begin;
    for (; kt + STAGES - 1 <= kt_last; kt += STAGES) static_for<STAGES>([&](auto st) { step(kt + st, st); });
    static_for<STAGES>([&](auto st) {
        if (kt + st <= kt_last) step(kt + st, st);
    });

    if constexpr (SPLITK > 1) {
        // wavefronts 1..3 park their partial sums; wavefront 0 adds them in order 1, 2, 3
        constexpr int PER_WAVE = NM * JB * 16 * kWave;
        if (wave > 0) {
            static_for<NM>([&](auto i) {
                static_for<JB>([&](auto j) {
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        red[(wave - 1) * PER_WAVE + ((i * JB + j) * 16 + v) * kWave + lane] = acc[i][j][v];
                });
            });
        }
        __syncthreads();
        if (wave > 0) return;
        for (int w = 0; w < SPLITK - 1; ++w) {
            static_for<NM>([&](auto i) {
                static_for<JB>([&](auto j) {
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        acc[i][j][v] += red[w * PER_WAVE + ((i * JB + j) * 16 + v) * kWave + lane];
                });
            });
        }
    }
    static_for<JB>([&](auto j) {
        const int tr = j * 32 + li;
        const bool live = tr < t.rows;
        store_block<GATEUP>(acc[0][j], acc[GATEUP ? 1 : 0][j], a.Out + (size_t)(t.row0 + (live ? tr : 0)) * a.ldo, n0w,
                            half, N, live);
    });
}

// =============================================================================================
// launch helpers
// =============================================================================================
// k-loop rotation between the workgroups of an XCD, in steps.  Single-block experts (weights
// streamed once): 2, which spreads the row-strided token tile reads over the L2 channels.
// Multi-tile experts (the LDS-DMA kernels): 0, so that row tiles that share a weight panel, and
// feature tiles that share a token tile, walk k together and meet in L2 (measured: a third
// fewer L2 misses, ~3 % faster at Mixtral T=4096).
inline int rot_steps(bool dma) {
    const int v = knob(kKnobRot);
    return v >= 0 ? v : (dma ? 0 : 2);
}


template <int IB, bool GATEUP, int STAGES, int XD, bool PACKED, bool WNT>
hipError_t launch_tile(const GemmArgs& a, int max_blocks, hipStream_t s) {
    constexpr int BN = 4 * IB * 32;
    constexpr int lds = 2 * 256 * kLdsStride * (int)sizeof(uint16_t);   // two buffers of 256 padded rows: 72 KiB
    auto kern = tile_kernel<IB, GATEUP, STAGES, XD, PACKED, WNT>;
    // dynamic LDS above 64 KB needs an explicit opt-in; once per process and kernel (not allowed
    // while a stream is being captured into a graph)
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (attr != hipSuccess) return attr;
    GemmArgs args = a;
    args.n_tiles_n = (a.N + BN - 1) / BN;
    const long long grid = (long long)max_blocks * args.n_tiles_n;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kThreads), lds, s, args);
    return hipGetLastError();
}

// Launch order switches, feature-tile count and grid of a tile_kernel_mixed launch (host arithmetic
// only; `cus` = CUs of the device).  Returns the grid size.
template <int IB, bool GATEUP, bool WNT>
inline long long mixed_launch_shape(GemmArgs& args, int max_blocks, int cus) {
    constexpr int BN = 4 * IB * 32;
    args.n_tiles_n = (args.N + BN - 1) / BN;
    args.rot_mul = rot_steps(false);
    // Test knobs (see moe_internal.hpp) can override the three launch-order choices; -1 = the rule.
    args.sib = knob(kKnobSideBySide) >= 0 ? knob(kKnobSideBySide) : 1;
    args.even = knob(kKnobEvenRows) >= 0 ? knob(kKnobEvenRows) : (GATEUP ? 1 : 2);
    args.chunk = knob(kKnobXcdChunk) >= 0 ? knob(kKnobXcdChunk) : (!GATEUP && WNT ? 1 : 0);
    args.no_nt = knob(kKnobNoNt) > 0;
    args.short_nt = knob(kKnobShortNt) >= 0 ? knob(kKnobShortNt) : (GATEUP ? 64 : 0);
    args.rot_mul_multi = rot_steps(true);
    long long grid = ((long long)max_blocks * args.n_tiles_n + 7) / 8 * 8;   // whole eighths for the per-XCD chunking
    args.slots = 0;
    if constexpr (IB == 2 && !GATEUP) {
        args.slots = cus;
        grid += cus / 2;     // a split last round has up to slots/2 extra workgroups
    }
    return grid;
}

template <int IB, bool GATEUP, bool PACKED, bool WNT, bool HALF = false>
hipError_t launch_tile_mixed(const GemmArgs& a, int max_blocks, hipStream_t s) {
    constexpr int lds = 4 * (HALF ? 4 : 8) * 32 * 128;   // the DMA ring: XD+1 = 4 buffers of 256 (128) rows x 128 bytes
    auto kern = tile_kernel_mixed<IB, GATEUP, PACKED, WNT, HALF>;
    // once per process and kernel: not allowed while a stream is being captured into a graph
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (attr != hipSuccess) return attr;
    static const int cus = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess) return 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        return n;
    }();
    GemmArgs args = a;
    const long long grid = mixed_launch_shape<IB, GATEUP, WNT>(args, max_blocks, cus);
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kThreads), lds, s, args);
    return hipGetLastError();
}

template <int JB, bool GATEUP, int STAGES, int SPLITK, bool PACKED>
hipError_t launch_skinny(const GemmArgs& a, int max_blocks, hipStream_t s) {
    constexpr int BN = (SPLITK == 1) ? 128 : 32;
    GemmArgs args = a;
    args.n_tiles_n = (a.N + BN - 1) / BN;
    const long long grid = (long long)max_blocks * args.n_tiles_n;
    hipLaunchKernelGGL((skinny_kernel<JB, GATEUP, STAGES, SPLITK, PACKED>), dim3((unsigned)grid), dim3(kThreads), 0,
                       s, args);
    return hipGetLastError();
}

struct Variant {
    int M;          // tallest block (Alg. 1's M) this variant can hold; it serves any schedule with M <= this
    bool packed;    // consumes moe_pack_weights' layout
    launch_fn fn;
    const char* name;   // kernel template instance, as rocprofv3 prints it (minus namespaces)
};

// A test may force a variant by table index through a knob; the index is ignored unless that
// variant matches the tile height and weight layout in use.
inline int forced_variant(int which, int count, int M, bool packed, const Variant* table) {
    const int id = knob(which);
    return (id >= 0 && id < count && table[id].M >= M && table[id].packed == packed) ? id : -1;
}

}  // namespace

}  // namespace moe
