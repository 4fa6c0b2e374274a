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
// From half a million logits on (and more than 8 experts) the fp64 work is cut down to the experts that can
// be among the k largest: a first pass computes every logit on the bf16 matrix cores with a
// proven error bound, the top-k pass takes the experts within twice that bound of the k-th
// largest value as candidates (k of them plus, rarely, one or two) and recomputes their logits
// exactly in fp64 before it selects.  Same indices, same order, same weights to ~1e-7 as the
// all-fp64 path at a third of its time (DeepSeek-V3 shape, T=4096); see fast_logits_kernel.
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

// ---- kernel 1, fast form: all logits on the bf16 matrix cores, with an error bound ----------
// One wavefront per unit of 32 tokens x NB*32 experts x one slice of d, v_mfma_f32_32x32x16_bf16
// with the token rows as the first operand: lane l supplies, per MFMA, 8 reduction elements of
// token row l%32 and of expert row l%32, and receives D[token 8(v/4) + 4(l/32) + v%4][expert l%32].
// The reduction runs in groups of 64 elements: lane half h = l/32 loads the 32 consecutive
// elements h*32.. of the group (64 contiguous bytes) and the j-th MFMA of the group takes its
// j-th 16-byte piece; both operands use the same assignment, so the sum is the same.  The four
// MFMAs of a group accumulate in fp32; the group's sum is then added to fp64 accumulators.
//
// Error bound.  bf16 products are exact in fp32.  Taking each MFMA's result (16 products plus
// the accumulator) to be off by at most 2^-19 of the sum of the magnitudes involved (32 units in
// the last place of the largest term: room for truncation and for a multi-stage adder), a group of
// four is off by at most 2^-17 * S_g, S_g = sum over the group of |x_k w_k|; the conversions and
// the fp64 additions add ~1e-16.  So
//     |z_fast - z| <= 2^-17 * sum_k |x_k w_k| <= 2^-17 * |x_t|_2 * |w_e|_2.
// The units of the first token tile also leave sum_k w_ek^2 per expert and slice (fp32) for that.
// part[ks][t][e], t < T32*32, e < E32*32 (fp64); wsq[ks][e] (fp32).
template <int NB>
__global__ __launch_bounds__(kThreads) void fast_logits_kernel(const uint16_t* __restrict__ x,
                                                              const uint16_t* __restrict__ wr,
                                                              double* __restrict__ part, float* __restrict__ wsq,
                                                              int T, int d, int E, int T32, int E32, int KS,
                                                              int units) {
    const int lane = threadIdx.x % kWave;
    const int unit = blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
    if (unit >= units) return;
    const int EG = (E32 + NB - 1) / NB;
    const int ks = unit % KS;
    const int eg = (unit / KS) % EG;
    const int tt = unit / (KS * EG);
    const int r = lane & 31, h = lane >> 5;
    const int ngroup = d / 64;
    const int per = (ngroup + KS - 1) / KS;
    const int g0 = ks * per;
    const int g1 = (g0 + per) < ngroup ? (g0 + per) : ngroup;

    const int trow = (tt * 32 + r) < T ? (tt * 32 + r) : (T - 1);
    const uint16_t* xp = x + (size_t)trow * d + h * 32;
    const uint16_t* wp[NB];
#pragma unroll
    for (int n = 0; n < NB; ++n) {
        const int erow = ((eg * NB + n) * 32 + r) < E ? ((eg * NB + n) * 32 + r) : (E - 1);
        wp[n] = wr + (size_t)erow * d + h * 32;
    }
    double acc[NB][16];
    float sq[NB];
#pragma unroll
    for (int n = 0; n < NB; ++n) {
        sq[n] = 0.0f;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[n][v] = 0.0;
    }
    if (g0 < g1) {
        uint4 xa[4], wb[NB][4];
        auto load = [&](int g, uint4 (&xo)[4], uint4 (&wo)[NB][4]) {
#pragma unroll
            for (int j = 0; j < 4; ++j) xo[j] = *reinterpret_cast<const uint4*>(xp + (size_t)g * 64 + j * 8);
#pragma unroll
            for (int n = 0; n < NB; ++n)
#pragma unroll
                for (int j = 0; j < 4; ++j) wo[n][j] = *reinterpret_cast<const uint4*>(wp[n] + (size_t)g * 64 + j * 8);
        };
        load(g0, xa, wb);
        for (int g = g0; g < g1; ++g) {
            uint4 xn[4], wn[NB][4];
            load(g + 1 < g1 ? g + 1 : g, xn, wn);   // prefetch (the last group re-reads itself)
#pragma unroll
            for (int n = 0; n < NB; ++n) {
                f32x16 c;
#pragma unroll
                for (int v = 0; v < 16; ++v) c[v] = 0.0f;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, xa[j]),
                                                                __builtin_bit_cast(bf16x8, wb[n][j]), c, 0, 0, 0);
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[n][v] += (double)c[v];
                if (tt == 0) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const uint32_t w4[4] = {wb[n][j].x, wb[n][j].y, wb[n][j].z, wb[n][j].w};
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float lo = __uint_as_float(w4[i] << 16), hi = __uint_as_float(w4[i] & 0xffff0000u);
                            sq[n] = fmaf(lo, lo, fmaf(hi, hi, sq[n]));
                        }
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) xa[j] = xn[j];
#pragma unroll
            for (int n = 0; n < NB; ++n)
#pragma unroll
                for (int j = 0; j < 4; ++j) wb[n][j] = wn[n][j];
        }
    }
    const size_t EP = (size_t)E32 * 32;
#pragma unroll
    for (int n = 0; n < NB; ++n) {
        const int et = eg * NB + n;
        if (et < E32) {
            double* out = part + ((size_t)ks * T32 * 32 + (size_t)tt * 32) * EP + (size_t)et * 32 + r;
#pragma unroll
            for (int v = 0; v < 16; ++v) out[(size_t)(8 * (v / 4) + 4 * h + v % 4) * EP] = acc[n][v];
            if (tt == 0) {
                const float both = sq[n] + __shfl_xor(sq[n], 32, kWave);
                if (h == 0) wsq[(size_t)ks * EP + (size_t)et * 32 + r] = both;
            }
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

// The logits of the experts that can be among the k largest, recomputed exactly (see
// fast_logits_kernel for the bound).  z holds the fast logits (bias included); on return the
// candidates' entries are exact: dot product in fp64 (bf16 operands and their products are
// exact there; the order of the additions moves the sum by ~1e-15), plus the bias.
// Why this is enough: let b = 2^-17 |x_t| max_e |w_e| >= every |z_fast - z|, and v_k the k-th
// largest fast value.  The k experts with the largest fast values have true logits >= v_k - b, so
// the true k-th largest logit is >= v_k - b, every expert of the true top-k has z >= v_k - b and
// therefore z_fast >= v_k - 2b: it is a candidate.  Every non-candidate has z <= z_fast + b <
// v_k - b, i.e. lies below k candidates' exact values, also when it keeps its fast value: the
// selection over the mixed array picks the same experts in the same order as over exact logits.
// The softmax denominator takes the non-candidates' fast values (relative error of a weight
// ~1e-7 at most: their scores weigh in with the error bound times their share).
// cand_list: LDS, kMaxExperts ints per wavefront.
__device__ __forceinline__ void refine_candidates(double (&z)[kLogitsPerLane], const bool (&ok)[kLogitsPerLane],
                                                  int lane, int t, int k, int E, int d, int KS, size_t EP,
                                                  const uint16_t* __restrict__ x, const uint16_t* __restrict__ wr,
                                                  const float* __restrict__ bias, const float* __restrict__ wsq,
                                                  int32_t* cand_list) {
    constexpr int Q = kLogitsPerLane;
    constexpr int CB = 12;  // candidates recomputed per pass over the token row (k = 8 gives 8, 9, rarely 10)
    const double ninf = -__builtin_huge_val();
    const uint16_t* xr = x + (size_t)t * d;
    // |x_t|^2 (fp32: squares of bf16 are exact, the sum is good to 1e-6 relative) and max_e |w_e|^2
    float xs = 0.0f;
    for (int p = lane; p < d / 8; p += kWave) {
        const uint4 v = *reinterpret_cast<const uint4*>(xr + (size_t)p * 8);
        const uint32_t w4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float lo = __uint_as_float(w4[i] << 16), hi = __uint_as_float(w4[i] & 0xffff0000u);
            xs = fmaf(lo, lo, fmaf(hi, hi, xs));
        }
    }
    float wm = 0.0f;
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const int e = lane + kWave * q;
        if (ok[q]) {
            float sum = 0.0f;
            for (int s0 = 0; s0 < KS; ++s0) sum += wsq[(size_t)s0 * EP + e];
            wm = fmaxf(wm, sum);
        }
    }
    const double x2 = wave_sum((double)xs), w2 = wave_max((double)wm);
    // twice the bound, with 1 % for the rounding of the two norms; NaN or inf makes every expert a candidate
    const double margin = 2.02 * 0x1p-17 * sqrt(x2 * w2);
    // k-th largest fast value
    unsigned taken = 0;
    double vk = ninf;
    for (int r = 0; r < k; ++r) {
        double bv = ninf;
        int bq = -1;
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            if (ok[q] && !((taken >> q) & 1u) && (bq < 0 || z[q] > bv)) {
                bv = z[q];
                bq = q;
            }
        }
        int be = bq < 0 ? -1 : lane + kWave * bq;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const double ov = __shfl_xor(bv, off, kWave);
            const int oe = __shfl_xor(be, off, kWave);
            if (oe >= 0 && (be < 0 || ov > bv || (ov == bv && oe < be))) {
                bv = ov;
                be = oe;
            }
        }
        if (be >= 0 && lane == be % kWave) taken |= 1u << (be / kWave);
        vk = bv;
    }
    // candidate list (ascending expert index inside each q; the order does not matter)
    int n_cand = 0;
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const bool c = ok[q] && !(z[q] < vk - margin);   // written so that a NaN anywhere keeps the expert in
        const unsigned long long bal = __ballot(c);
        if (c) cand_list[n_cand + __popcll(bal & ((1ull << lane) - 1ull))] = lane + kWave * q;
        n_cand += __popcll(bal);
    }
    __builtin_amdgcn_wave_barrier();
    for (int c0 = 0; c0 < n_cand; c0 += CB) {
        int ce[CB];
#pragma unroll
        for (int b = 0; b < CB; ++b) ce[b] = *(volatile int32_t*)&cand_list[(c0 + b < n_cand) ? c0 + b : c0];
        double acc[CB];
#pragma unroll
        for (int b = 0; b < CB; ++b) acc[b] = 0.0;
        for (int p = lane; p < d / 8; p += kWave) {
            double xv[8];
            unpack8(*reinterpret_cast<const uint4*>(xr + (size_t)p * 8), xv);
            uint4 wv[CB];
#pragma unroll
            for (int b = 0; b < CB; ++b)   // the condition is uniform over the wavefront: unused slots cost nothing
                if (c0 + b < n_cand) wv[b] = *reinterpret_cast<const uint4*>(wr + (size_t)ce[b] * d + (size_t)p * 8);
#pragma unroll
            for (int b = 0; b < CB; ++b) {
                if (c0 + b < n_cand) {
                    double w8[8];
                    unpack8(wv[b], w8);
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[b] = fma(xv[j], w8[j], acc[b]);
                }
            }
        }
#pragma unroll
        for (int b = 0; b < CB; ++b) {
            if (c0 + b < n_cand) {   // uniform over the wavefront
                const double tot = wave_sum(acc[b]) + (bias ? (double)bias[ce[b]] : 0.0);
                if (lane == ce[b] % kWave) {
#pragma unroll
                    for (int q = 0; q < Q; ++q) z[q] = (q == ce[b] / kWave) ? tot : z[q];
                }
            }
        }
    }
}

// ---- kernel 2: gate + top-k, one wavefront per token ------------------------------------------
// FAST: `part` holds the fast logits' slices (row tiles of 32, see fast_logits_kernel), refined here.
template <bool FAST>
__global__ __launch_bounds__(kThreads) void topk_kernel(const double* __restrict__ part,
                                                       const float* __restrict__ bias,
                                                       int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
                                                       int T, int E, int k, int gating, int T16, int E16, int KS,
                                                       int32_t* __restrict__ zero, int zero_n,
                                                       const uint16_t* __restrict__ x, const uint16_t* __restrict__ wr,
                                                       int d, const float* __restrict__ wsq) {
    __shared__ double wsel[kWavesPerBlock][kMaxExperts];
    __shared__ int32_t sel_idx[kWavesPerBlock][kMaxExperts];
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int t = blockIdx.x * kWavesPerBlock + wave;
    if (t >= T) return;
    zero_token_counters(zero, zero_n, t, lane);

    constexpr int Q = kLogitsPerLane;
    const double ninf = -__builtin_huge_val();
    const size_t EP = (size_t)E16 * 16;   // (FAST: T16 and E16 are passed as twice the 32-tile counts)
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
    if constexpr (FAST) refine_candidates(z, ok, lane, t, k, E, d, KS, EP, x, wr, bias, wsq, sel_idx[wave]);
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
    bool fast;          // bf16 logits + exact candidates; then T16/E16 count 16-row units of the 32-padded sizes
    int T32, E32, NB;
};

// mode: the test knob's value.  -1 the rule, 1 every logit in fp64, 0 the bf16 first pass from 256 tokens on.
RoutePlan plan(const moe_config& c, int mode) {
    RoutePlan p;
    // From half a million logits on (DeepSeek-V3 shape: 2048 tokens); below, the exact pass over
    // ~k+1 router rows per token costs more than the fp64 matrix cores need for all of them
    // (measured: Qwen2-MoE shape T=4096 72 -> 104 us, DeepSeek-V3 shape T=512 57 -> 86 us).
    p.fast = mode != 1 && c.E > 8 && (mode == 0 ? c.T >= 256 : (long long)c.T * c.E >= (1ll << 19));
    if (p.fast) {
        p.T32 = (c.T + 31) / 32;
        p.E32 = (c.E + 31) / 32;
        p.T16 = 2 * p.T32;
        p.E16 = 2 * p.E32;
        p.NB = p.E32 >= 4 ? 4 : (p.E32 >= 2 ? 2 : 1);
        p.NT = 0;
        const long long tiles = (long long)p.T32 * ((p.E32 + p.NB - 1) / p.NB);
        const int ngroup = c.d / 64;
        long long ks = (1024 + tiles - 1) / tiles;          // one wavefront per SIMD or more
        if (ks > 16) ks = 16;
        if (ks > ngroup / 2) ks = ngroup / 2;
        if (ks < 1) ks = 1;
        p.KS = (int)ks;
        return p;
    }
    p.T32 = p.E32 = p.NB = 0;
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
    // sized for whichever form a test knob may switch to
    size_t need = 0;
    for (int mode = -1; mode <= 1; ++mode) {
        const RoutePlan p = plan(c, mode);
        size_t bytes = (size_t)p.KS * p.T16 * 16 * p.E16 * 16 * sizeof(double);
        if (p.fast) bytes += (size_t)p.KS * p.E16 * 16 * sizeof(float);
        need = bytes > need ? bytes : need;
    }
    return need;
}

hipError_t launch_route(const moe_config& c, const uint16_t* x, const uint16_t* wr, const float* bias,
                        int32_t* topk_idx, float* topk_w, void* workspace, int32_t* zero, int zero_per_token, hipStream_t s) {
    if (c.E <= 8 && c.T <= 2048) {   // measured: with 16 experts or more tokens the MFMA path is faster
        const dim3 g(c.T);
        hipLaunchKernelGGL(route_direct_kernel<8>, g, dim3(kThreads), 0, s, x, wr, bias, topk_idx, topk_w, c.d, c.E,
                           c.k, c.gating, zero, zero_per_token);
        return hipGetLastError();
    }
    const RoutePlan p = plan(c, knob(kKnobRouteExact));
    if (p.fast) {
        const int units = p.T32 * ((p.E32 + p.NB - 1) / p.NB) * p.KS;
        double* part = (double*)workspace;
        float* wsq = (float*)(part + (size_t)p.KS * p.T32 * 32 * p.E32 * 32);
        const dim3 grid((units + kWavesPerBlock - 1) / kWavesPerBlock);
        auto go = [&](auto kern) {
            hipLaunchKernelGGL(kern, grid, dim3(kThreads), 0, s, x, wr, part, wsq, c.T, c.d, c.E, p.T32, p.E32, p.KS, units);
        };
        if (p.NB == 4) go(fast_logits_kernel<4>);
        else if (p.NB == 2) go(fast_logits_kernel<2>);
        else go(fast_logits_kernel<1>);
        hipLaunchKernelGGL(topk_kernel<true>, dim3((c.T + kWavesPerBlock - 1) / kWavesPerBlock), dim3(kThreads), 0, s,
                           part, bias, topk_idx, topk_w, c.T, c.E, c.k, c.gating, p.T16, p.E16, p.KS, zero, zero_per_token,
                           x, wr, c.d, wsq);
        return hipGetLastError();
    }
    const int units = p.T16 * ((p.E16 + p.NT - 1) / p.NT) * p.KS;
    double* part = (double*)workspace;
    const dim3 grid((units + kWavesPerBlock - 1) / kWavesPerBlock);
    if (p.NT == 4)
        hipLaunchKernelGGL(logits_kernel<4>, grid, dim3(kThreads), 0, s, x, wr, part, c.T, c.d, c.E, p.T16, p.E16,
                           p.KS, units);
    else
        hipLaunchKernelGGL(logits_kernel<1>, grid, dim3(kThreads), 0, s, x, wr, part, c.T, c.d, c.E, p.T16, p.E16,
                           p.KS, units);
    hipLaunchKernelGGL(topk_kernel<false>, dim3((c.T + kWavesPerBlock - 1) / kWavesPerBlock), dim3(kThreads), 0, s, part,
                       bias, topk_idx, topk_w, c.T, c.E, c.k, c.gating, p.T16, p.E16, p.KS, zero, zero_per_token,
                       nullptr, nullptr, 0, nullptr);
    return hipGetLastError();
}

}  // namespace moe
