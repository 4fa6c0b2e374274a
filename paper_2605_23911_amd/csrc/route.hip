// Router: logits z = W_r x (+ bias) in fp64 on the fp64 matrix cores, then softmax / sigmoid
// gate and a wavefront top-k.
// Paper: Eq. 1 and Eq. 2 (Sec. 2.1); Sec. 3.4 (max-subtracted softmax, iterative arg-max with
// the winner masked, softmax and sigmoid gating).  Unlike the paper the projection is part of
// this stage (no library GEMM), and the arg-max runs on the logits with an explicit
// "already chosen" mask instead of overwriting scores with -1.
//
// Why fp64: the expert indices must equal those of an exact evaluation.  With hundreds of
// experts and thousands of tokens the smallest gap between neighbouring top-(k+1) logits is of
// the order of 1e-6, below what an fp32-accumulated dot product of length d resolves.  bf16
// operands convert exactly to fp64 and their products are exact there, so the fp64 MFMA
// (v_mfma_f64_16x16x4) gives logits good to ~1e-15 at the fp64 matrix rate.
//
// Kernel 1 (logits): one wavefront per work unit (16 tokens x 16 experts x one slice of d).
//   The reduction is cut into enough slices to put >= ~2000 wavefronts on the chip even for
//   one token and eight experts; each unit writes its 16x16 fp64 partial tile.
// Kernel 2 (gate + top-k): one wavefront per token sums the slices, applies the gate and
//   selects k experts.
// Models with at most 8 experts take a single kernel instead (route_direct_kernel).
#include "moe_internal.hpp"

namespace moe {

namespace {

typedef double f64x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kWavesPerBlock = kThreads / kWave;
constexpr int kChunk = 32;   // reduction elements per chunk: 4 lane groups x 8 consecutive k

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

__device__ __forceinline__ double wave_max(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmax(v, __shfl_xor(v, off, kWave));
    return v;
}

__device__ __forceinline__ void unpack8(const uint4& v, double* out) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        out[2 * i] = (double)__uint_as_float(w[i] << 16);
        out[2 * i + 1] = (double)__uint_as_float(w[i] & 0xffff0000u);
    }
}

// ---- kernel 1: partial logit tiles ----------------------------------------------------------
// part[ks][t][e], t < T16*16, e < E16*16 (padded to whole tiles).
// MFMA operand layout (v_mfma_f64_16x16x4): lane l supplies A[i = l%16][k = l/16] and
// B[k = l/16][j = l%16]; it receives D[i = l/16 + 4v][j = l%16], v = 0..3.  The MFMA sums over
// k, so which k a slot carries is free as long as A and B agree: lane group g = l/16 loads 8
// consecutive k (one 16-byte load) and the q-th MFMA of a chunk takes element q of every lane.
// NT: 16-expert tiles per wavefront (1 or 4).  With 4 the token fragment is loaded and
// converted once per chunk for 64 experts (used when there are enough tiles to fill the chip
// without cutting the reduction).
template <int NT>
__global__ __launch_bounds__(kThreads) void logits_kernel(const uint16_t* __restrict__ x,
                                                         const uint16_t* __restrict__ wr,
                                                         double* __restrict__ part, int T, int d, int E, int T16,
                                                         int E16, int KS, int units) {
    const int lane = threadIdx.x % kWave;
    const int unit = blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
    if (unit >= units) return;
    const int EG = (E16 + NT - 1) / NT;   // expert-tile groups
    const int ks = unit % KS;
    const int eg = (unit / KS) % EG;
    const int tt = unit / (KS * EG);
    const int i = lane & 15, g = lane >> 4;

    const int nchunk = d / kChunk;
    const int per = (nchunk + KS - 1) / KS;
    const int c0 = ks * per;
    const int c1 = (c0 + per) < nchunk ? (c0 + per) : nchunk;

    const int trow = (tt * 16 + i) < T ? (tt * 16 + i) : (T - 1);
    const uint16_t* xp = x + (size_t)trow * d + g * 8;
    const uint16_t* wp[NT];
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        const int erow = ((eg * NT + n) * 16 + i) < E ? ((eg * NT + n) * 16 + i) : (E - 1);
        wp[n] = wr + (size_t)erow * d + g * 8;
    }

    f64x4 acc[NT];
#pragma unroll
    for (int n = 0; n < NT; ++n) acc[n] = f64x4{0.0, 0.0, 0.0, 0.0};
    if (c0 < c1) {
        uint4 xr = *reinterpret_cast<const uint4*>(xp + (size_t)c0 * kChunk);
        uint4 wv[NT];
#pragma unroll
        for (int n = 0; n < NT; ++n) wv[n] = *reinterpret_cast<const uint4*>(wp[n] + (size_t)c0 * kChunk);
        for (int c = c0; c < c1; ++c) {
            const int cn = (c + 1 < c1) ? c + 1 : c;   // prefetch (the last chunk re-reads itself)
            const uint4 xn = *reinterpret_cast<const uint4*>(xp + (size_t)cn * kChunk);
            uint4 wn[NT];
#pragma unroll
            for (int n = 0; n < NT; ++n) wn[n] = *reinterpret_cast<const uint4*>(wp[n] + (size_t)cn * kChunk);
            double a8[8];
            unpack8(xr, a8);
#pragma unroll
            for (int n = 0; n < NT; ++n) {
                double b8[8];
                unpack8(wv[n], b8);
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    acc[n] = __builtin_amdgcn_mfma_f64_16x16x4f64(a8[q], b8[q], acc[n], 0, 0, 0);
            }
            xr = xn;
#pragma unroll
            for (int n = 0; n < NT; ++n) wv[n] = wn[n];
        }
    }
    const size_t EP = (size_t)E16 * 16;
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        const int et = eg * NT + n;
        if (et < E16) {
            double* out = part + ((size_t)ks * T16 * 16 + (size_t)tt * 16) * EP + (size_t)et * 16 + i;
#pragma unroll
            for (int v = 0; v < 4; ++v) out[(size_t)(g + 4 * v) * EP] = acc[n][v];
        }
    }
}

// ---- gate + top-k of one token by one wavefront ---------------------------------------------
// Lane l holds the logits of experts l, l+64, ... in z[] (ok[] = expert exists).  Eq. 1-2,
// Sec. 3.4: max-subtracted softmax (or sigmoid), k rounds of arg-max over the logits with the
// winners masked, ties to the lower index.
constexpr int kLogitsPerLane = kMaxExperts / kWave;
// moe_forward's down projection counts, per (token, 128-feature group), how many of the token's
// k expert rows have been written (see ffn_kernels.hpp, fused_combine).  The counters of token t
// are cleared here by the wavefront that routes t, so the layer needs no clearing launch.
__device__ __forceinline__ void zero_token_counters(int32_t* __restrict__ zero, int zero_n, int t, int lane) {
    if (zero == nullptr) return;
    for (int i = lane; i < zero_n; i += kWave) zero[(size_t)t * zero_n + i] = 0;
}

__device__ __forceinline__ void gate_and_select(double (&z)[kLogitsPerLane], const bool (&ok)[kLogitsPerLane],
                                                int lane, int wave, int t, int k, int gating,
                                                double (*wsel)[kMaxExperts], int32_t (*sel_idx)[kMaxExperts],
                                                int32_t* __restrict__ topk_idx, float* __restrict__ topk_w) {
    constexpr int Q = kLogitsPerLane;
    const double ninf = -__builtin_huge_val();
    double p[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) z[q] = (z[q] != z[q]) ? ninf : z[q];   // a NaN logit can never win and never breaks the index range
    double m = ninf;
#pragma unroll
    for (int q = 0; q < Q; ++q) m = fmax(m, z[q]);
    m = wave_max(m);
    double psum = 0.0;
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        if (gating == MOE_GATE_SIGMOID_NORM)
            p[q] = ok[q] ? 1.0 / (1.0 + exp(-z[q])) : 0.0;
        else
            p[q] = ok[q] ? exp(z[q] - m) : 0.0;
        psum += p[q];
    }
    psum = wave_sum(psum);
    if (gating != MOE_GATE_SIGMOID_NORM) {
        const double inv = 1.0 / psum;
#pragma unroll
        for (int q = 0; q < Q; ++q) p[q] = ok[q] ? p[q] * inv : 0.0;   // softmax scores, Eq. 1
    }

    unsigned taken = 0;   // bit q set: this lane's q-th expert already selected
    double wsum = 0.0;
    for (int r = 0; r < k; ++r) {
        double bv = ninf;
        int be = -1;
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            if (ok[q] && !((taken >> q) & 1u) && (be < 0 || z[q] > bv)) {
                bv = z[q];
                be = lane + kWave * q;
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const double ov = __shfl_xor(bv, off, kWave);
            const int oe = __shfl_xor(be, off, kWave);
            if (oe >= 0 && (be < 0 || ov > bv || (ov == bv && oe < be))) {
                bv = ov;
                be = oe;
            }
        }
        // every lane now holds the same winner `be` (ties resolved to the lower index)
        const int oq = be / kWave, ol = be % kWave;
        double mine = 0.0;
#pragma unroll
        for (int q = 0; q < Q; ++q) mine = (q == oq) ? p[q] : mine;
        const double wv = __shfl(mine, ol, kWave);
        if (lane == ol) taken |= 1u << oq;
        wsum += wv;
        if (lane == 0) {
            sel_idx[wave][r] = be;
            wsel[wave][r] = wv;
        }
    }
    const double scale = (gating == MOE_GATE_SOFTMAX) ? 1.0 : 1.0 / wsum;
    __builtin_amdgcn_wave_barrier();
    for (int i = lane; i < k; i += kWave) {
        topk_idx[(size_t)t * k + i] = *(volatile int32_t*)&sel_idx[wave][i];
        topk_w[(size_t)t * k + i] = (float)(*(volatile double*)&wsel[wave][i] * scale);
    }
}

// ---- kernel 2: gate + top-k, one wavefront per token ------------------------------------------
__global__ __launch_bounds__(kThreads) void topk_kernel(const double* __restrict__ part,
                                                       const float* __restrict__ bias,
                                                       int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
                                                       int T, int E, int k, int gating, int T16, int E16, int KS,
                                                       int32_t* __restrict__ zero, int zero_n) {
    __shared__ double wsel[kWavesPerBlock][kMaxExperts];
    __shared__ int32_t sel_idx[kWavesPerBlock][kMaxExperts];
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int t = blockIdx.x * kWavesPerBlock + wave;
    if (t >= T) return;
    zero_token_counters(zero, zero_n, t, lane);

    constexpr int Q = kLogitsPerLane;
    const double ninf = -__builtin_huge_val();
    const size_t EP = (size_t)E16 * 16;
    double z[Q];
    bool ok[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const int e = lane + kWave * q;
        ok[q] = e < E;
        double v = ninf;
        if (ok[q]) {
            v = bias ? (double)bias[e] : 0.0;
            for (int s0 = 0; s0 < KS; s0 += 8) {   // slices in fixed order; 8 independent loads at a time
                double tmp[8];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    tmp[u] = (s0 + u < KS) ? part[((size_t)(s0 + u) * T16 * 16 + t) * EP + e] : 0.0;
#pragma unroll
                for (int u = 0; u < 8; ++u) v += tmp[u];
            }
        }
        z[q] = v;
    }
    gate_and_select(z, ok, lane, wave, t, k, gating, wsel, sel_idx, topk_idx, topk_w);
}

// ---- few experts (E <= 8): the whole router in one kernel, one workgroup per token ----------
// With 8 experts a 16x16 MFMA tile would be half padding and the two-kernel path costs
// two launches for a few microseconds of work.  Here thread i takes 8 consecutive k of every
// 2048, multiplies them with the same k of all E router rows in fp64 (bf16 -> fp64 is exact, so
// are the products); butterfly sums and one LDS exchange leave the logits in wavefront 0, which
// applies the gate and selects.  All loads of a thread are issued before the first use.
template <int EB>
__global__ __launch_bounds__(kThreads) void route_direct_kernel(const uint16_t* __restrict__ x,
                                                               const uint16_t* __restrict__ wr,
                                                               const float* __restrict__ bias,
                                                               int32_t* __restrict__ topk_idx,
                                                               float* __restrict__ topk_w, int d, int E, int k,
                                                               int gating, int32_t* __restrict__ zero, int zero_n) {
    __shared__ double wsel[kWavesPerBlock][kMaxExperts];
    __shared__ int32_t sel_idx[kWavesPerBlock][kMaxExperts];
    __shared__ double partial[kWavesPerBlock][EB];
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int t = blockIdx.x;
    double acc[EB];
#pragma unroll
    for (int e = 0; e < EB; ++e) acc[e] = 0.0;
    const uint16_t* xr = x + (size_t)t * d;
    for (int k0 = threadIdx.x * 8; k0 < d; k0 += 2 * kThreads * 8) {
        // two chunks per trip (the second clamped to the first when it falls beyond d)
        const int k1 = k0 + kThreads * 8;
        const bool two = k1 < d;
        const int k1c = two ? k1 : k0;
        uint4 xa = *reinterpret_cast<const uint4*>(xr + k0), xb = *reinterpret_cast<const uint4*>(xr + k1c);
        uint4 wa[EB], wb[EB];
#pragma unroll
        for (int e = 0; e < EB; ++e) {   // rows beyond E re-read the last row; their sums are never used
            const uint16_t* row = wr + (size_t)(e < E ? e : E - 1) * d;
            wa[e] = *reinterpret_cast<const uint4*>(row + k0);
            wb[e] = *reinterpret_cast<const uint4*>(row + k1c);
        }
        double xv[8], yv[8];
        unpack8(xa, xv);
        unpack8(xb, yv);
#pragma unroll
        for (int e = 0; e < EB; ++e) {
            double w8[8];
            unpack8(wa[e], w8);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[e] = fma(xv[j], w8[j], acc[e]);
            unpack8(wb[e], w8);
            double a2 = 0.0;
#pragma unroll
            for (int j = 0; j < 8; ++j) a2 = fma(yv[j], w8[j], a2);
            acc[e] += two ? a2 : 0.0;
        }
    }
#pragma unroll
    for (int e = 0; e < EB; ++e) {
        const double tot = wave_sum(acc[e]);
        if (lane == 0) partial[wave][e] = tot;
    }
    __syncthreads();
    if (wave != 0) return;
    zero_token_counters(zero, zero_n, t, lane);
    constexpr int Q = kLogitsPerLane;
    double z[Q];
    bool ok[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        ok[q] = q == 0 && lane < E;
        z[q] = -__builtin_huge_val();
    }
    if (ok[0]) {
        double v = bias ? (double)bias[lane] : 0.0;
#pragma unroll
        for (int w = 0; w < kWavesPerBlock; ++w) v += partial[w][lane];
        z[0] = v;
    }
    gate_and_select(z, ok, lane, 0, t, k, gating, wsel, sel_idx, topk_idx, topk_w);
}

struct RoutePlan {
    int T16, E16, KS, NT;
};

RoutePlan plan(const moe_config& c) {
    RoutePlan p;
    p.T16 = (c.T + 15) / 16;
    p.E16 = (c.E + 15) / 16;
    // four expert tiles per wavefront (the converted token fragment is then shared by 64 experts)
    // from 64 such units on; the reduction is cut further to keep ~2000 wavefronts (measured:
    // Qwen2-MoE shape T=4096 85 -> 67 us, DeepSeek-V3 shape T=512 66 -> 57 us)
    p.NT = (p.E16 >= 4 && (long long)p.T16 * ((p.E16 + 3) / 4) >= 64) ? 4 : 1;
    const long long tiles = (long long)p.T16 * ((p.E16 + p.NT - 1) / p.NT);
    const int nchunk = c.d / kChunk;
    long long ks = (2048 + tiles - 1) / tiles;          // aim for >= ~2048 wavefronts
    if (ks > 16) ks = 16;                               // the top-k kernel sums the slices serially
    if (ks > nchunk / 2) ks = nchunk / 2;               // at least two chunks per slice
    if (ks < 1) ks = 1;
    p.KS = (int)ks;
    return p;
}

}  // namespace

size_t route_workspace_bytes(const moe_config& c) {
    if (c.T == 0) return 0;
    const RoutePlan p = plan(c);
    return (size_t)p.KS * p.T16 * 16 * p.E16 * 16 * sizeof(double);
}

hipError_t launch_route(const moe_config& c, const uint16_t* x, const uint16_t* wr, const float* bias,
                        int32_t* topk_idx, float* topk_w, void* workspace, int32_t* zero, int zero_per_token, hipStream_t s) {
    if (c.E <= 8 && c.T <= 2048) {   // measured: with 16 experts or more tokens the MFMA path is faster
        const dim3 g(c.T);
        hipLaunchKernelGGL(route_direct_kernel<8>, g, dim3(kThreads), 0, s, x, wr, bias, topk_idx, topk_w, c.d, c.E,
                           c.k, c.gating, zero, zero_per_token);
        return hipGetLastError();
    }
    const RoutePlan p = plan(c);
    const int units = p.T16 * ((p.E16 + p.NT - 1) / p.NT) * p.KS;
    double* part = (double*)workspace;
    const dim3 grid((units + kWavesPerBlock - 1) / kWavesPerBlock);
    if (p.NT == 4)
        hipLaunchKernelGGL(logits_kernel<4>, grid, dim3(kThreads), 0, s, x, wr, part, c.T, c.d, c.E, p.T16, p.E16,
                           p.KS, units);
    else
        hipLaunchKernelGGL(logits_kernel<1>, grid, dim3(kThreads), 0, s, x, wr, part, c.T, c.d, c.E, p.T16, p.E16,
                           p.KS, units);
    hipLaunchKernelGGL(topk_kernel, dim3((c.T + kWavesPerBlock - 1) / kWavesPerBlock), dim3(kThreads), 0, s, part,
                       bias, topk_idx, topk_w, c.T, c.E, c.k, c.gating, p.T16, p.E16, p.KS, zero, zero_per_token);
    return hipGetLastError();
}

}  // namespace moe
