// Stand-alone measurement, not part of the library: what rate of v_mfma_f32_32x32x16_bf16 does
// this MI355X sustain when nothing but the matrix cores is in the way?
//
// The GEMM kernels of this package run one wavefront per SIMD, 256 workgroups of 4 wavefronts on
// 256 CUs; so does this probe.  Every wavefront issues MFMAs back to back on 16 independent
// accumulators (no instruction waits for a result).  Three register-only runs differ in the
// operand bits only: zeros, constants, random bf16 values with exponents like those of N(0,1)
// activations; a fourth run feeds the token operand from LDS at the GEMM bodies' ratio (one
// ds_read_b128 per two MFMAs).  The shader clock is read from the cycle counter against the
// constant 100 MHz counter: the chip lowers it under load, and the load depends on how many bits
// toggle, i.e. on the data.  The published dense bf16 peak (2.5 PFLOP/s) is 1024 FLOP per cycle
// and SIMD at 2.4 GHz.
//
// build: hipcc -O3 --offload-arch=gfx950 -o mfma_ceiling_probe mfma_ceiling_probe.hip   (done by __graft_entry__.build())
// run:   ./mfma_ceiling_probe
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <vector>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define CHECK(x)                                                                          \
    do {                                                                                  \
        hipError_t e_ = (x);                                                              \
        if (e_ != hipSuccess) {                                                           \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);    \
            std::exit(1);                                                                 \
        }                                                                                 \
    } while (0)

constexpr int kWorkgroups = 256, kThreads = 256, kAcc = 16;
constexpr double kFlopPerMfma = 2.0 * 32 * 32 * 16;

enum Operands { kZeros = 0, kConstants = 1, kRandom = 2 };

__device__ inline unsigned mix(unsigned x) {
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}
// random sign and mantissa, exponent 2^-2 .. 2^0: the bulk of a unit normal's bit patterns
__device__ inline unsigned short random_bf16(unsigned& state) {
    const unsigned h = mix(state += 0x9e3779b9u);
    return (unsigned short)((h & 0x807f) | ((125 + ((h >> 8) % 3)) << 7));
}

struct Clocks { unsigned long long shader, fixed; };   // elapsed shader cycles / 100 MHz ticks of wavefront 0

// Register-only: 4 weight-side and 4 token-side fragments, 16 accumulators.
__global__ __launch_bounds__(kThreads) void registers_only(float* out, int mfmas_per_acc, int operands, Clocks* clk) {
    bf16x8 a[4], b[4];
    unsigned state = (blockIdx.x * kThreads + threadIdx.x) * 977u + 1;
    for (int n = 0; n < 4; ++n)
        for (int i = 0; i < 8; ++i) {
            unsigned short ua = 0, ub = 0;
            if (operands == kConstants) { ua = 0x3f80; ub = 0x4000; }
            if (operands == kRandom) { ua = random_bf16(state); ub = random_bf16(state); }
            a[n][i] = __builtin_bit_cast(__bf16, ua);
            b[n][i] = __builtin_bit_cast(__bf16, ub);
        }
    f32x16 acc[kAcc];
    for (int n = 0; n < kAcc; ++n)
        for (int v = 0; v < 16; ++v) acc[n][v] = 0.f;
    const unsigned long long c0 = __builtin_readcyclecounter(), r0 = wall_clock64();
    for (int it = 0; it < mfmas_per_acc; it += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int n = 0; n < kAcc; ++n)
                acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[n % 4], b[(n / 2 + u) % 4], acc[n], 0, 0, 0);
        }
    }
    const unsigned long long c1 = __builtin_readcyclecounter(), r1 = wall_clock64();
    float s = 0;
    for (int n = 0; n < kAcc; ++n)
        for (int v = 0; v < 16; ++v) s += acc[n][v];
    out[blockIdx.x * kThreads + threadIdx.x] = s;
    if (threadIdx.x == 0) clk[blockIdx.x] = Clocks{c1 - c0, r1 - r0};
}

// Token fragments from LDS (two buffers of 256 rows x 64 k, rows padded to 72 elements), weight
// fragments in registers; per step of 64 k: 4 x 8 ds_read_b128 and 4 x 16 MFMAs per wavefront,
// as in the GEMM bodies at 256 rows.
__global__ __launch_bounds__(kThreads) void tokens_from_lds(float* out, int steps, Clocks* clk) {
    constexpr int kStride = 72, kBuf = 256 * kStride;
    __shared__ __attribute__((aligned(16))) unsigned short lds[2 * kBuf];
    unsigned state = (blockIdx.x * kThreads + threadIdx.x) * 977u + 1;
    for (int i = threadIdx.x; i < 2 * kBuf; i += kThreads) lds[i] = random_bf16(state);
    bf16x8 a[8];
    for (int n = 0; n < 8; ++n)
        for (int i = 0; i < 8; ++i) a[n][i] = __builtin_bit_cast(__bf16, random_bf16(state));
    __syncthreads();
    f32x16 acc[kAcc];
    for (int n = 0; n < kAcc; ++n)
        for (int v = 0; v < 16; ++v) acc[n][v] = 0.f;
    const int lane = threadIdx.x % 64;
    const int rd = (lane & 31) * kStride + (lane >> 5) * 8;
    const unsigned long long c0 = __builtin_readcyclecounter(), r0 = wall_clock64();
    for (int it = 0; it < steps; ++it) {
        const int buf = (it & 1) * kBuf;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            bf16x8 xf[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) xf[j] = *reinterpret_cast<const bf16x8*>(&lds[buf + rd + j * 32 * kStride + s * 16]);
#pragma unroll
            for (int i = 0; i < 2; ++i) {
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    acc[i * 8 + j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s * 2 + i], xf[j], acc[i * 8 + j], 0, 0, 0);
            }
        }
    }
    const unsigned long long c1 = __builtin_readcyclecounter(), r1 = wall_clock64();
    float s = 0;
    for (int n = 0; n < kAcc; ++n)
        for (int v = 0; v < 16; ++v) s += acc[n][v];
    out[blockIdx.x * kThreads + threadIdx.x] = s;
    if (threadIdx.x == 0) clk[blockIdx.x] = Clocks{c1 - c0, r1 - r0};
}

static void report(const char* what, float ms, double mfmas_per_wavefront, const std::vector<Clocks>& h) {
    double cycles = 0, ticks = 0;
    for (const Clocks& c : h) { cycles += (double)c.shader; ticks += (double)c.fixed; }
    const double flop = (double)kWorkgroups * 4 * mfmas_per_wavefront * kFlopPerMfma;
    const double rate = flop / (ms * 1e-3);
    std::printf("%-52s %7.2f ms  %6.3f PFLOP/s = %.3f of 2.5  shader clock %4.0f MHz  %.1f cycles per MFMA\n", what, ms,
                rate / 1e15, rate / 2.5e15, cycles / ticks * 100.0, cycles / kWorkgroups / mfmas_per_wavefront);
    std::fflush(stdout);
}

int main() {
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    float* out;
    Clocks* clk;
    CHECK(hipMalloc(&out, sizeof(float) * kWorkgroups * kThreads));
    CHECK(hipMalloc(&clk, sizeof(Clocks) * kWorkgroups));
    std::vector<Clocks> h(kWorkgroups);
    float ms;
    std::printf("v_mfma_f32_32x32x16_bf16, %d workgroups x 4 wavefronts, one wavefront per SIMD (about 10 ms per run)\n", kWorkgroups);
    const char* names[] = {"registers only, operands all zero", "registers only, operands constant (1.0, 2.0)",
                           "registers only, operands random bf16"};
    for (int rep = 0; rep < 2; ++rep) {
        for (int operands = 0; operands < 3; ++operands) {
            const int per_acc = 40000;
            hipLaunchKernelGGL(registers_only, dim3(kWorkgroups), dim3(kThreads), 0, 0, out, 1000, operands, clk);   // warm-up
            CHECK(hipDeviceSynchronize());
            CHECK(hipEventRecord(e0));
            hipLaunchKernelGGL(registers_only, dim3(kWorkgroups), dim3(kThreads), 0, 0, out, per_acc, operands, clk);
            CHECK(hipEventRecord(e1));
            CHECK(hipEventSynchronize(e1));
            CHECK(hipGetLastError());
            CHECK(hipEventElapsedTime(&ms, e0, e1));
            CHECK(hipMemcpy(h.data(), clk, sizeof(Clocks) * kWorkgroups, hipMemcpyDeviceToHost));
            report(names[operands], ms, (double)per_acc * kAcc, h);
        }
        const int steps = 10000;
        hipLaunchKernelGGL(tokens_from_lds, dim3(kWorkgroups), dim3(kThreads), 0, 0, out, 1000, clk);   // warm-up
        CHECK(hipDeviceSynchronize());
        CHECK(hipEventRecord(e0));
        hipLaunchKernelGGL(tokens_from_lds, dim3(kWorkgroups), dim3(kThreads), 0, 0, out, steps, clk);
        CHECK(hipEventRecord(e1));
        CHECK(hipEventSynchronize(e1));
        CHECK(hipGetLastError());
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        CHECK(hipMemcpy(h.data(), clk, sizeof(Clocks) * kWorkgroups, hipMemcpyDeviceToHost));
        report("token operand from LDS (1 ds_read_b128 : 2 MFMA), random", ms, (double)steps * 64, h);
    }
    CHECK(hipFree(out));
    CHECK(hipFree(clk));
    return 0;
}
