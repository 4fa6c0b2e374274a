// Router: logits z = W_r x (+ bias) in fp64, softmax / sigmoid gate, wavefront top-k.
// Paper: Eq. 1 and Eq. 2 (Sec. 2.1); Sec. 3.4 (max-subtracted softmax, iterative arg-max
// with the winner masked, softmax and sigmoid gating).  Unlike the paper the projection is
// part of this kernel, and the arg-max runs on the logits with an explicit "already chosen"
// mask instead of overwriting scores with -1.
#include "moe_internal.hpp"

namespace moe {

namespace {

constexpr int kRouteTokens = 4;   // tokens per workgroup == wavefronts per workgroup
constexpr int kRouteDC = 2048;    // elements of d staged in LDS per pass
constexpr int kRouteThreads = kRouteTokens * kWave;

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

__global__ __launch_bounds__(kRouteThreads) void route_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ wr, const float* __restrict__ bias,
    int32_t* __restrict__ topk_idx, float* __restrict__ topk_w, int T, int d, int E, int k, int gating) {
    __shared__ uint4 xs[kRouteTokens][kRouteDC / 8];
    __shared__ double zs[kRouteTokens][kMaxExperts];
    __shared__ int32_t sel_idx[kRouteTokens][kMaxExperts];

    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int t0 = blockIdx.x * kRouteTokens;

    for (int i = tid; i < kRouteTokens * E; i += kRouteThreads) {
        const int e = i % E;
        zs[i / E][e] = bias ? (double)bias[e] : 0.0;
    }

    // ---- logits: every wavefront owns the experts e = wave (mod 4); lanes stride over d.
    for (int c0 = 0; c0 < d; c0 += kRouteDC) {
        const int cv = ((d - c0) < kRouteDC ? (d - c0) : kRouteDC) / 8;   // 16-byte vectors in this pass
        __syncthreads();
        for (int v = tid; v < kRouteTokens * cv; v += kRouteThreads) {
            const int tt = v / cv, j = v % cv;
            const int t = (t0 + tt < T) ? (t0 + tt) : (T - 1);
            xs[tt][j] = *reinterpret_cast<const uint4*>(x + (size_t)t * d + c0 + j * 8);
        }
        __syncthreads();
        for (int e = wave; e < E; e += kRouteTokens) {
            double acc[kRouteTokens];
#pragma unroll
            for (int tt = 0; tt < kRouteTokens; ++tt) acc[tt] = 0.0;
            const uint16_t* wrow = wr + (size_t)e * d + c0;
            for (int j = lane; j < cv; j += kWave) {
                double w8[8];
                unpack8(*reinterpret_cast<const uint4*>(wrow + j * 8), w8);
#pragma unroll
                for (int tt = 0; tt < kRouteTokens; ++tt) {
                    double x8[8];
                    unpack8(xs[tt][j], x8);
#pragma unroll
                    for (int q = 0; q < 8; ++q) acc[tt] = fma(x8[q], w8[q], acc[tt]);
                }
            }
#pragma unroll
            for (int tt = 0; tt < kRouteTokens; ++tt) acc[tt] = wave_sum(acc[tt]);
            if (lane == 0) {
#pragma unroll
                for (int tt = 0; tt < kRouteTokens; ++tt) zs[tt][e] += acc[tt];
            }
        }
    }
    __syncthreads();

    // ---- gate + top-k: wavefront `wave` finishes token t0 + wave.
    const int t = t0 + wave;
    if (t >= T) return;

    constexpr int Q = kMaxExperts / kWave;   // logits per lane
    const double ninf = -__builtin_huge_val();
    double z[Q], p[Q];
    bool ok[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const int e = lane + kWave * q;
        ok[q] = e < E;
        double v = ok[q] ? zs[wave][e] : ninf;
        z[q] = (v != v) ? ninf : v;   // a NaN logit can never win and never breaks the index range
    }
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
            zs[wave][r] = wv;   // the logit row lives in registers by now; reuse its LDS row
        }
    }
    const double scale = (gating == MOE_GATE_SOFTMAX) ? 1.0 : 1.0 / wsum;
    __builtin_amdgcn_wave_barrier();
    for (int i = lane; i < k; i += kWave) {
        topk_idx[(size_t)t * k + i] = *(volatile int32_t*)&sel_idx[wave][i];
        topk_w[(size_t)t * k + i] = (float)(*(volatile double*)&zs[wave][i] * scale);
    }
}

}  // namespace

hipError_t launch_route(const moe_config& c, const uint16_t* x, const uint16_t* wr, const float* bias,
                        int32_t* topk_idx, float* topk_w, hipStream_t s) {
    const int grid = (c.T + kRouteTokens - 1) / kRouteTokens;
    hipLaunchKernelGGL(route_kernel, dim3(grid), dim3(kRouteThreads), 0, s, x, wr, bias, topk_idx, topk_w,
                       c.T, c.d, c.E, c.k, c.gating);
    return hipGetLastError();
}

}  // namespace moe
