// Permutation into expert-contiguous order and the block schedule, all on the device.
// Paper: Sec. 2.2 (n_e), Sec. 3.5 (stable sort by expert + row gather), Sec. 3.2 Algorithm 1
// (block schedule).  The paper sorts with a library call and builds the schedule on the host
// behind a device->host sync (its limitation 2); here a three-kernel counting sort keeps
// everything on the stream: per-chunk histograms, one scan, per-chunk stable ranks.
#include <mutex>

#include "moe_internal.hpp"

namespace moe {

namespace {

// Chunk histograms for moe_permute_static, the entry point for callers that cannot allocate:
// one array per GPU, held from the moment the library's code object is loaded on that GPU until
// the process ends.  In host code the name below is only a handle for hipGetSymbolAddress: the
// kernels are given the device address that call returns, never the name.
constexpr size_t kStaticScratchInts = MOE_PERMUTE_STATIC_MAX_INTS;
static __device__ __align__(256) int32_t scratch[kStaticScratchInts];

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;

// An expert id outside [0, E) cannot be reported without a device->host sync; it is clamped
// (identically in every kernel) so that no destination row ever leaves the buffers.
__device__ __forceinline__ int clamp_expert(int e, int E) { return e < 0 ? 0 : (e >= E ? E - 1 : e); }

// ---- 1. per-chunk histogram -------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void hist_kernel(const int32_t* __restrict__ topk_idx, int R, int E,
                                                       int32_t* __restrict__ chunk_counts) {
    __shared__ int32_t hist[kMaxExperts];
    const int tid = threadIdx.x;
    hist[tid] = 0;
    __syncthreads();
    const int j0 = blockIdx.x * kPermChunk;
    for (int j = j0 + tid; j < j0 + kPermChunk && j < R; j += kThreads)
        atomicAdd(&hist[clamp_expert(topk_idx[j], E)], 1);
    __syncthreads();
    if (tid < E) chunk_counts[(size_t)blockIdx.x * E + tid] = hist[tid];
}

// Exclusive scan of one value per thread over a 256-thread workgroup; returns the exclusive
// prefix and leaves the grand total in *total (LDS).
__device__ __forceinline__ int block_exclusive_scan(int v, int* wave_tot, int* total) {
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    int inc = v;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const int o = __shfl_up(inc, off, kWave);
        if (lane >= off) inc += o;
    }
    if (lane == kWave - 1) wave_tot[wave] = inc;
    __syncthreads();
    int base = 0;
    for (int w = 0; w < wave; ++w) base += wave_tot[w];
    if (tid == kThreads - 1) *total = base + inc;
    __syncthreads();
    return base + inc - v;
}

// Owner of block q in a list where expert e's blocks start at first[e] (non-decreasing in e):
// the last expert whose first block index is <= q (experts that contribute no block share a
// start with their successor, so the last one is the owner).
__device__ __forceinline__ int owner_of_block(const int* first, int n, int q) {
    int lo = 0, hi = n - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (first[mid] <= q) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// Algorithm 1: expert e contributes ceil(n_e / M) blocks (e, b*M), experts in ascending order.
// Runs on one 256-thread workgroup; `n_e` is this thread's expert count (0 for tid >= E).
// blocks_mix != nullptr asks for a second list with the same blocks as a stable partition: first
// those of the experts that span several blocks (n_e > M, "heavy": their workgroups are bound by
// the matrix cores), then the others ("light": bound by the weight stream), each class in
// ascending expert order; *num_heavy = blocks of the first class.  The down projection deals the
// two classes evenly over its launch (see tile_kernel_mixed).
__device__ __forceinline__ void emit_block_schedule(int n_e, int M, int32_t* __restrict__ blocks,
                                                    int32_t* __restrict__ num_blocks,
                                                    int32_t* __restrict__ blocks_mix,
                                                    int32_t* __restrict__ num_heavy, int* first, int* first2,
                                                    int* wave_tot, int* total) {
    const int tid = threadIdx.x;
    const int nb = (n_e + M - 1) / M;
    const int excl = block_exclusive_scan(nb, wave_tot, total);
    first[tid] = excl;
    __syncthreads();
    const int nblk = *total;
    if (tid == 0) *num_blocks = nblk;
    for (int q = tid; q < nblk; q += kThreads) {
        const int e = owner_of_block(first, kThreads, q);
        blocks[2 * q] = e;
        blocks[2 * q + 1] = (q - first[e]) * M;
    }
    if (blocks_mix == nullptr) return;
    __syncthreads();
    const bool heavy = nb > 1;
    const int excl_h = block_exclusive_scan(heavy ? nb : 0, wave_tot, total);
    const int n_heavy = *total;
    __syncthreads();
    const int excl_l = block_exclusive_scan(heavy ? 0 : nb, wave_tot, total);
    first[tid] = excl_h;
    first2[tid] = excl_l;
    __syncthreads();
    if (tid == 0) *num_heavy = n_heavy;
    for (int q = tid; q < nblk; q += kThreads) {
        int e, b;
        if (q < n_heavy) {
            e = owner_of_block(first, kThreads, q);
            b = q - first[e];
        } else {
            e = owner_of_block(first2, kThreads, q - n_heavy);
            b = q - n_heavy - first2[e];
        }
        blocks_mix[2 * q] = e;
        blocks_mix[2 * q + 1] = b * M;
    }
}

// ---- 2. scan: chunk bases, counts, offsets, block schedule --------------------------------
// chunk_counts[c][e] is replaced by the first destination row of expert e's slots in chunk c.
__global__ __launch_bounds__(kThreads) void scan_kernel(int32_t* __restrict__ chunk_counts, int nchunks, int E,
                                                       int R, int32_t* __restrict__ counts,
                                                       int32_t* __restrict__ offsets, int M,
                                                       int32_t* __restrict__ blocks,
                                                       int32_t* __restrict__ num_blocks,
                                                       int32_t* __restrict__ blocks_mix,
                                                       int32_t* __restrict__ num_heavy) {
    __shared__ int wave_tot[kWaves];
    __shared__ int total;
    __shared__ int first[kThreads], first2[kThreads];
    const int tid = threadIdx.x;
    int n_e = 0;
    if (tid < E)
        for (int c = 0; c < nchunks; ++c) n_e += chunk_counts[(size_t)c * E + tid];
    const int off = block_exclusive_scan(n_e, wave_tot, &total);
    if (tid < E) {
        counts[tid] = n_e;
        offsets[tid] = off;
        int run = off;
        for (int c = 0; c < nchunks; ++c) {
            const int v = chunk_counts[(size_t)c * E + tid];
            chunk_counts[(size_t)c * E + tid] = run;
            run += v;
        }
    }
    if (tid == 0) offsets[E] = R;
    if (blocks != nullptr) {
        __syncthreads();
        emit_block_schedule(n_e, M, blocks, num_blocks, blocks_mix, num_heavy, first, first2, wave_tot, &total);
    }
}

__global__ __launch_bounds__(kThreads) void schedule_kernel(const int32_t* __restrict__ offsets, int E, int M,
                                                           int32_t* __restrict__ blocks,
                                                           int32_t* __restrict__ num_blocks,
                                                           int32_t* __restrict__ blocks_mix,
                                                           int32_t* __restrict__ num_heavy) {
    __shared__ int wave_tot[kWaves];
    __shared__ int total;
    __shared__ int first[kThreads], first2[kThreads];
    const int tid = threadIdx.x;
    const int n_e = tid < E ? offsets[tid + 1] - offsets[tid] : 0;
    emit_block_schedule(n_e, M, blocks, num_blocks, blocks_mix, num_heavy, first, first2, wave_tot, &total);
}

// ---- 3. stable rank -----------------------------------------------------------------------
// Each wavefront owns 256 consecutive slots of the chunk and walks them 64 at a time in slot
// order; within a group the rank among equal experts is the number of lower lanes holding the
// same expert, so equal experts keep their slot order (stable).
__global__ __launch_bounds__(kThreads) void rank_kernel(const int32_t* __restrict__ topk_idx, int R, int E,
                                                       const int32_t* __restrict__ chunk_base,
                                                       int32_t* __restrict__ row_of,
                                                       int32_t* __restrict__ src_of) {
    __shared__ int32_t wcnt[kWaves][kMaxExperts];
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    constexpr int kPerWave = kPermChunk / kWaves;
    constexpr int kGroups = kPerWave / kWave;
    for (int w = 0; w < kWaves; ++w) wcnt[w][tid] = 0;
    __syncthreads();
    const int jw = blockIdx.x * kPermChunk + wave * kPerWave;
    int e_of[kGroups];
#pragma unroll
    for (int g = 0; g < kGroups; ++g) {
        const int j = jw + g * kWave + lane;
        e_of[g] = j < R ? clamp_expert(topk_idx[j], E) : -1;
        if (e_of[g] >= 0) atomicAdd(&wcnt[wave][e_of[g]], 1);
    }
    __syncthreads();
    if (tid < E) {   // counts per wavefront -> first destination row per wavefront
        int run = chunk_base[(size_t)blockIdx.x * E + tid];
        for (int w = 0; w < kWaves; ++w) {
            const int v = wcnt[w][tid];
            wcnt[w][tid] = run;
            run += v;
        }
    }
    __syncthreads();
    volatile int32_t* next = wcnt[wave];
#pragma unroll
    for (int g = 0; g < kGroups; ++g) {
        const int e = e_of[g];
        // lanes holding the same expert id: AND over the 8 id bits of agreeing ballots
        unsigned long long same = __ballot(e >= 0);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const unsigned long long bal = __ballot((e >> b) & 1);
            same &= ((e >> b) & 1) ? bal : ~bal;
        }
        if (e >= 0) {
            const unsigned long long below = same & ((1ull << lane) - 1ull);
            const int base = next[e];
            const int r = base + __popcll(below);
            const int j = jw + g * kWave + lane;
            row_of[j] = r;
            src_of[r] = j;
            if (below == 0) next[e] = base + __popcll(same);   // lowest lane of the set advances it
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// ---- 1+2+3 in one workgroup, for up to 8192 slots (every batch of a few hundred tokens) -----
// Same counting sort, run by one 1024-thread workgroup: launch latency, not work, is what the
// three-kernel version costs at this size.  Wavefront w owns slots [w*P, (w+1)*P), P = 64*G.
constexpr int kFusedThreads = 1024;
constexpr int kFusedWaves = kFusedThreads / kWave;
constexpr int kFusedMaxGroups = 8;
constexpr int kFusedMaxSlots = kFusedWaves * kFusedMaxGroups * kWave;

// Exclusive scan of v[0..255] (LDS) by wavefront 0 into out[0..255]; returns the total in *total.
__device__ __forceinline__ void wave0_scan256(const int* v, int* out, int* total, int lane) {
    const int a0 = v[4 * lane], a1 = v[4 * lane + 1], a2 = v[4 * lane + 2], a3 = v[4 * lane + 3];
    const int sum = a0 + a1 + a2 + a3;
    int inc = sum;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const int o = __shfl_up(inc, off, kWave);
        if (lane >= off) inc += o;
    }
    const int ex = inc - sum;
    out[4 * lane] = ex;
    out[4 * lane + 1] = ex + a0;
    out[4 * lane + 2] = ex + a0 + a1;
    out[4 * lane + 3] = ex + a0 + a1 + a2;
    if (lane == kWave - 1) *total = inc;
}

__global__ __launch_bounds__(kFusedThreads) void fused_permute_kernel(
    const int32_t* __restrict__ topk_idx, int R, int E, int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
    int32_t* __restrict__ row_of, int32_t* __restrict__ src_of, int M, int32_t* __restrict__ blocks,
    int32_t* __restrict__ num_blocks, int32_t* __restrict__ blocks_mix, int32_t* __restrict__ num_heavy) {
    __shared__ int32_t wcnt[kFusedWaves][kMaxExperts];
    __shared__ int cnt[kMaxExperts], off[kMaxExperts], nb[kMaxExperts], first[kMaxExperts];
    __shared__ int nbh[kMaxExperts], firsth[kMaxExperts], nbl[kMaxExperts], firstl[kMaxExperts];
    __shared__ int total_rows, total_blocks, total_heavy, total_light;
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int G = (R + kFusedWaves * kWave - 1) / (kFusedWaves * kWave);   // 64-slot groups per wavefront
    const int jw = wave * G * kWave;

    for (int i = tid; i < kFusedWaves * kMaxExperts; i += kFusedThreads) (&wcnt[0][0])[i] = 0;
    __syncthreads();
    int e_of[kFusedMaxGroups];
#pragma unroll
    for (int g = 0; g < kFusedMaxGroups; ++g) {
        const int j = jw + g * kWave + lane;
        e_of[g] = (g < G && j < R) ? clamp_expert(topk_idx[j], E) : -1;
        if (e_of[g] >= 0) atomicAdd(&wcnt[wave][e_of[g]], 1);
    }
    __syncthreads();
    if (tid < kMaxExperts) {
        int n = 0;
        if (tid < E)
            for (int w = 0; w < kFusedWaves; ++w) n += wcnt[w][tid];
        cnt[tid] = n;
        // block counts per expert: all (Algorithm 1's list), and split by class for the second
        // list (see emit_block_schedule): multi-block experts in nbh, the others in nbl
        const int b = (n + M - 1) / M;
        nb[tid] = b;
        nbh[tid] = b > 1 ? b : 0;
        nbl[tid] = b > 1 ? 0 : b;
    }
    __syncthreads();
    if (wave == 0) {
        wave0_scan256(cnt, off, &total_rows, lane);
        wave0_scan256(nb, first, &total_blocks, lane);
        if (blocks_mix != nullptr) {
            wave0_scan256(nbh, firsth, &total_heavy, lane);
            wave0_scan256(nbl, firstl, &total_light, lane);
        }
    }
    __syncthreads();
    if (tid < E) {
        counts[tid] = cnt[tid];
        offsets[tid] = off[tid];
        int run = off[tid];
        for (int w = 0; w < kFusedWaves; ++w) {
            const int v = wcnt[w][tid];
            wcnt[w][tid] = run;
            run += v;
        }
    }
    if (tid == 0) offsets[E] = R;
    if (blocks != nullptr) {   // Algorithm 1 and its heavy-first partition, as in emit_block_schedule
        const int nblk = total_blocks;
        if (tid == 0) *num_blocks = nblk;
        for (int q = tid; q < nblk; q += kFusedThreads) {
            const int e = owner_of_block(first, kMaxExperts, q);
            blocks[2 * q] = e;
            blocks[2 * q + 1] = (q - first[e]) * M;
        }
        if (blocks_mix != nullptr) {
            const int n1 = total_heavy;
            if (tid == 0) *num_heavy = n1;
            for (int q = tid; q < nblk; q += kFusedThreads) {
                int e, b;
                if (q < n1) {
                    e = owner_of_block(firsth, kMaxExperts, q);
                    b = q - firsth[e];
                } else {
                    e = owner_of_block(firstl, kMaxExperts, q - n1);
                    b = q - n1 - firstl[e];
                }
                blocks_mix[2 * q] = e;
                blocks_mix[2 * q + 1] = b * M;
            }
        }
    }
    __syncthreads();
    volatile int32_t* next = wcnt[wave];
#pragma unroll
    for (int g = 0; g < kFusedMaxGroups; ++g) {
        if (g < G) {   // uniform over the workgroup
            const int e = e_of[g];
            unsigned long long same = __ballot(e >= 0);
#pragma unroll
            for (int b = 0; b < 8; ++b) {
                const unsigned long long bal = __ballot((e >> b) & 1);
                same &= ((e >> b) & 1) ? bal : ~bal;
            }
            if (e >= 0) {
                const unsigned long long below = same & ((1ull << lane) - 1ull);
                const int base = next[e];
                const int r = base + __popcll(below);
                const int j = jw + g * kWave + lane;
                row_of[j] = r;
                src_of[r] = j;
                if (below == 0) next[e] = base + __popcll(same);
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
}

// ---- 4. row gather ------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void gather_kernel(const uint16_t* __restrict__ x,
                                                         const int32_t* __restrict__ src_of, int k, int d,
                                                         uint16_t* __restrict__ x_perm, int ld_perm) {
    const int r = blockIdx.x;
    const int t = src_of[r] / k;
    const uint4* src = reinterpret_cast<const uint4*>(x + (size_t)t * d);
    uint4* dst = reinterpret_cast<uint4*>(x_perm + (size_t)r * ld_perm);
    for (int v = threadIdx.x; v < d / 8; v += kThreads) dst[v] = src[v];
}

}  // namespace

// Device address of this GPU's copy of `scratch`, looked up once per device (with that device
// current) and kept.  No allocation happens here or later.
hipError_t permute_static_scratch(int32_t** ptr) {
    constexpr int kMaxDevices = 64;
    static std::mutex lock;
    static int32_t* per_device[kMaxDevices] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(lock);
    if (per_device[dev] == nullptr) {
        int32_t* p = nullptr;
        e = hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        per_device[dev] = p;
    }
    *ptr = per_device[dev];
    return hipSuccess;
}

hipError_t launch_permute_index(const moe_config& c, const int32_t* topk_idx, int32_t* counts,
                                int32_t* offsets, int32_t* row_of, int32_t* src_of, int32_t* scratch,
                                int32_t M, int32_t* blocks, int32_t* num_blocks, int32_t* blocks_mix, int32_t* num_heavy,
                                hipStream_t s) {
    const int R = c.T * c.k;
    if (R <= kFusedMaxSlots) {
        hipLaunchKernelGGL(fused_permute_kernel, dim3(1), dim3(kFusedThreads), 0, s, topk_idx, R, c.E, counts,
                           offsets, row_of, src_of, M > 0 ? M : 1, blocks, num_blocks, blocks_mix, num_heavy);
        return hipGetLastError();
    }
    const int nchunks = permute_chunks(c);
    hipLaunchKernelGGL(hist_kernel, dim3(nchunks), dim3(kThreads), 0, s, topk_idx, R, c.E, scratch);
    hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(kThreads), 0, s, scratch, nchunks, c.E, R, counts, offsets, M,
                       blocks, num_blocks, blocks_mix, num_heavy);
    hipLaunchKernelGGL(rank_kernel, dim3(nchunks), dim3(kThreads), 0, s, topk_idx, R, c.E, scratch, row_of,
                       src_of);
    return hipGetLastError();
}

hipError_t launch_gather_rows(const moe_config& c, const uint16_t* x, const int32_t* src_of,
                              uint16_t* x_perm, int32_t ld_perm, hipStream_t s) {
    hipLaunchKernelGGL(gather_kernel, dim3(c.T * c.k), dim3(kThreads), 0, s, x, src_of, c.k, c.d, x_perm, ld_perm);
    return hipGetLastError();
}

hipError_t launch_block_schedule(const moe_config& c, const int32_t* offsets, int32_t M, int32_t* blocks,
                                 int32_t* num_blocks, int32_t* blocks_mix, int32_t* num_heavy, hipStream_t s) {
    hipLaunchKernelGGL(schedule_kernel, dim3(1), dim3(kThreads), 0, s, offsets, c.E, M, blocks, num_blocks,
                       blocks_mix, num_heavy);
    return hipGetLastError();
}

}  // namespace moe
