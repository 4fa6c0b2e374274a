// One-time re-ordering of the expert weights into the order the GEMM kernels' load
// instructions consume them (weights are static at inference).  Pure data movement: the
// packed buffer holds exactly the same bf16 values.
//
// Unit = 16 bytes (8 consecutive k of one weight row).  For a projection with N output rows
// and reduction length K the units are ordered
//     [expert][row block rb = row/32][k step kt = k/64][matrix m][slot s = 0..3][lane = 0..63]
// and unit (rb, kt, m, s, lane) holds  W_m[expert][rb*32 + lane%32][kt*64 + s*16 + (lane/32)*8 .. +8].
// gate and up (m = 0, 1) are interleaved per k step; the down projection has m = 0 only and
// follows the gate+up region.
#include "moe_internal.hpp"

namespace moe {

namespace {

__global__ __launch_bounds__(256) void pack_kernel(const uint16_t* __restrict__ w0, const uint16_t* __restrict__ w1,
                                                  uint16_t* __restrict__ out, int E, int N, int K, int NM) {
    const size_t units = (size_t)E * N * (K / 8) * NM;
    const int KT = K / 64, NRB = N / 32;
    for (size_t u = (size_t)blockIdx.x * blockDim.x + threadIdx.x; u < units; u += (size_t)gridDim.x * blockDim.x) {
        size_t r = u;
        const int lane = (int)(r % 64); r /= 64;
        const int s = (int)(r % 4); r /= 4;
        const int m = (int)(r % NM); r /= NM;
        const int kt = (int)(r % KT); r /= KT;
        const int rb = (int)(r % NRB); r /= NRB;
        const int e = (int)r;
        const uint16_t* src = (m == 0 ? w0 : w1) + ((size_t)e * N + rb * 32 + (lane & 31)) * K + kt * 64 + s * 16 +
                              (lane >> 5) * 8;
        reinterpret_cast<uint4*>(out)[u] = *reinterpret_cast<const uint4*>(src);
    }
}

}  // namespace

size_t packed_gate_up_bytes(const moe_config& c) { return (size_t)c.E * c.F * c.d * 2 * sizeof(uint16_t); }
size_t packed_down_bytes(const moe_config& c) { return (size_t)c.E * c.F * c.d * sizeof(uint16_t); }

hipError_t launch_pack(const moe_config& c, const uint16_t* wg, const uint16_t* wu, const uint16_t* wd,
                       uint16_t* packed, hipStream_t s) {
    uint16_t* gu = packed;
    uint16_t* dn = packed + packed_gate_up_bytes(c) / sizeof(uint16_t);
    hipLaunchKernelGGL(pack_kernel, dim3(256 * 16), dim3(256), 0, s, wg, wu, gu, c.E, c.F, c.d, 2);
    hipLaunchKernelGGL(pack_kernel, dim3(256 * 16), dim3(256), 0, s, wd, (const uint16_t*)nullptr, dn, c.E, c.d, c.F,
                       1);
    return hipGetLastError();
}

}  // namespace moe
