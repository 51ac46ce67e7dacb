// Device probe: what matrix rate and shader clock does this GPU sustain when the MFMA pipes are kept busy with the
// caller's operand bits and nothing else (no LDS, no memory traffic)?  The published peak of the part assumes its top
// clock; under a power cap the clock depends on how often the operand bits toggle, so the sustained figure is the
// one a GEMM on real data can be compared with.  Not part of the AGZO arithmetic.
#include "agzo_internal.h"

namespace agzo {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// One workgroup of 4 waves per CU.  Each lane keeps four A and four B fragments (8 bf16 each) taken from `operands`
// and sixteen 32x32 fp32 accumulators; an iteration is 8 groups of 16 MFMAs that cycle through the 16 fragment pairs.
// DUTY of the 8 groups are issued; the others are replaced by a sleep of about the same length.  (A compile-time
// DUTY: a run-time test per group costs about a tenth of the issue rate.)  DUTY = 9 issues the flop count of all 8
// groups as 16x16x32 instructions.
template <int DUTY>
__global__ __launch_bounds__(256) void probe_mfma_kernel(const uint4* __restrict__ operands, int iters,
                                                          unsigned long long* clk4, float* sink) {
    floatx16 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    bf16x8 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = __builtin_bit_cast(bf16x8, operands[i * 256 + threadIdx.x]);
        b[i] = __builtin_bit_cast(bf16x8, operands[(4 + i) * 256 + threadIdx.x]);
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) { clk4[0] = __builtin_readcyclecounter(); clk4[1] = wall_clock64(); }
    if constexpr (DUTY == 9) {
        // the same flop count per iteration from 16x16x32 instructions: 64 accumulators of four registers (a wave's
        // 128 x 128 tile), eight A and eight B fragments, every pair once per round, four rounds
        typedef float floatx4 __attribute__((ext_vector_type(4)));
        floatx4 c[64];
#pragma unroll
        for (int i = 0; i < 64; ++i) c[i] = floatx4{0.f, 0.f, 0.f, 0.f};
        bf16x8 a2[8], b2[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            a2[i] = __builtin_bit_cast(bf16x8, operands[((2 * i) & 7) * 256 + threadIdx.x]);
            b2[i] = __builtin_bit_cast(bf16x8, operands[((2 * i + 1) & 7) * 256 + threadIdx.x]);
        }
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int g = 0; g < 4; ++g)
#pragma unroll
                for (int i = 0; i < 64; ++i)
                    // (written out with the accumulator in the accumulation registers, as the GEMM has it: through the
                    // builtin these accumulators land in the ordinary registers, where the instruction issues at 0.81 of
                    // its rate)
                    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c[i]) : "v"(a2[((i >> 3) + g) & 7]), "v"(b2[((i & 7) + g) & 7]));
        }
#pragma unroll
        for (int i = 0; i < 64; ++i) acc[i & 15][i >> 4] += c[i][0] + c[i][1] + c[i][2] + c[i][3];
    } else
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            if (g < DUTY) {
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(i + g) & 3], b[((i >> 2) + g) & 3], acc[i], 0, 0, 0);
            } else {
                __builtin_amdgcn_s_sleep(8);
            }
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) { clk4[2] = __builtin_readcyclecounter(); clk4[3] = wall_clock64(); }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[i][e];
    if (s == 1.234e-30f) sink[threadIdx.x] = s;      // keeps the accumulators alive; never true for finite sums
}

hipError_t launch_probe_mfma(const void* operands, int duty, int iters, unsigned long long* clk4, hipStream_t st) {
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    const uint4* ops = static_cast<const uint4*>(operands);
    float* sink = reinterpret_cast<float*>(clk4 + 4);
    const dim3 grid((unsigned)cus), block(256);
    switch (duty) {
        case 1: hipLaunchKernelGGL(probe_mfma_kernel<1>, grid, block, 0, st, ops, iters, clk4, sink); break;
        case 2: hipLaunchKernelGGL(probe_mfma_kernel<2>, grid, block, 0, st, ops, iters, clk4, sink); break;
        case 3: hipLaunchKernelGGL(probe_mfma_kernel<3>, grid, block, 0, st, ops, iters, clk4, sink); break;
        case 4: hipLaunchKernelGGL(probe_mfma_kernel<4>, grid, block, 0, st, ops, iters, clk4, sink); break;
        case 5: hipLaunchKernelGGL(probe_mfma_kernel<5>, grid, block, 0, st, ops, iters, clk4, sink); break;
        case 6: hipLaunchKernelGGL(probe_mfma_kernel<6>, grid, block, 0, st, ops, iters, clk4, sink); break;
        case 7: hipLaunchKernelGGL(probe_mfma_kernel<7>, grid, block, 0, st, ops, iters, clk4, sink); break;
        case 8: hipLaunchKernelGGL(probe_mfma_kernel<8>, grid, block, 0, st, ops, iters, clk4, sink); break;
        case 9: hipLaunchKernelGGL(probe_mfma_kernel<9>, grid, block, 0, st, ops, iters, clk4, sink); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace agzo
