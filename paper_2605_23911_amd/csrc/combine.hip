// Un-permute + weighted combine: y[t,:] = sum_i w[t,i] * y_perm[row_of[t*k+i], :].
// Paper: Eq. 3, Sec. 3.5 (fp32 accumulation).  Written as a gather per output row instead
// of the paper's scatter: no atomics, fixed slot order, bit-reproducible.
#include "moe_internal.hpp"

namespace moe {

namespace {

constexpr int kThreads = 256;

__global__ __launch_bounds__(kThreads) void combine_kernel(const uint16_t* __restrict__ y_perm,
                                                          const int32_t* __restrict__ row_of,
                                                          const float* __restrict__ topk_w, int k, int d,
                                                          uint16_t* __restrict__ y) {
    const int t = blockIdx.x;
    const int32_t* rows = row_of + (size_t)t * k;
    const float* w = topk_w + (size_t)t * k;
    for (int c = threadIdx.x * 8; c < d; c += kThreads * 8) {
        float acc[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) acc[q] = 0.0f;
        for (int i = 0; i < k; ++i) {
            const uint4 v = *reinterpret_cast<const uint4*>(y_perm + (size_t)rows[i] * d + c);
            const float wi = w[i];
            const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                acc[2 * q] = fmaf(wi, __uint_as_float(u[q] << 16), acc[2 * q]);
                acc[2 * q + 1] = fmaf(wi, __uint_as_float(u[q] & 0xffff0000u), acc[2 * q + 1]);
            }
        }
        uint4 o;
        o.x = pack2_bf16(acc[0], acc[1]);
        o.y = pack2_bf16(acc[2], acc[3]);
        o.z = pack2_bf16(acc[4], acc[5]);
        o.w = pack2_bf16(acc[6], acc[7]);
        *reinterpret_cast<uint4*>(y + (size_t)t * d + c) = o;
    }
}

}  // namespace

hipError_t launch_combine(const moe_config& c, const uint16_t* y_perm, const int32_t* row_of,
                          const float* topk_w, uint16_t* y, hipStream_t s) {
    hipLaunchKernelGGL(combine_kernel, dim3(c.T), dim3(kThreads), 0, s, y_perm, row_of, topk_w, c.k, c.d, y);
    return hipGetLastError();
}

}  // namespace moe
