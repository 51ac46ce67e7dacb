// What sits between the linear layers of the gated-MLP stack workload (Alg. 2 over a model): RMS normalisation, the
// SiLU gate and the residual sum.  They are not steps of the method, only the model around it, but a whole-model step
// runs them three times per block, so they are single-pass kernels here: bf16 in and out, fp32 arithmetic, one
// rounding to bf16, 16-byte accesses.  All three are bound by HBM.
#include "agzo_internal.h"

namespace agzo {

__device__ __forceinline__ void unpack8(const uint4& v, float (&f)[8]) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = __uint_as_float(w[i] << 16);
        f[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
}
__device__ __forceinline__ uint4 pack8(const float (&f)[8]) {
    return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
}

// y[t][:] = gain * x[t][:] / sqrt(mean(x[t][:]^2) + eps); one workgroup per row, d a multiple of 8
__global__ __launch_bounds__(256) void glue_rmsnorm_kernel(const bf16_t* __restrict__ x, int64_t ldx, bf16_t* __restrict__ y,
                                                           int64_t ldy, const float* __restrict__ gain, int64_t d, float eps) {
    __shared__ float red[4];
    const int tid = threadIdx.x;
    const bf16_t* xr = x + (int64_t)blockIdx.x * ldx;
    bf16_t* yr = y + (int64_t)blockIdx.x * ldy;
    const int64_t nvec = d / 8;
    float ss = 0.f;
    for (int64_t v = tid; v < nvec; v += 256) {
        float f[8];
        unpack8(*reinterpret_cast<const uint4*>(xr + v * 8), f);
#pragma unroll
        for (int i = 0; i < 8; ++i) ss = fmaf(f[i], f[i], ss);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    const float scale = rsqrtf(((red[0] + red[1]) + (red[2] + red[3])) / (float)d + eps);
    for (int64_t v = tid; v < nvec; v += 256) {          // the row is re-read from cache
        float f[8];
        unpack8(*reinterpret_cast<const uint4*>(xr + v * 8), f);
#pragma unroll
        for (int i = 0; i < 8; ++i) f[i] = f[i] * scale * (gain ? gain[v * 8 + i] : 1.f);
        *reinterpret_cast<uint4*>(yr + v * 8) = pack8(f);
    }
}

// m = silu(a) * u, rows of d (multiple of 8) with leading dimensions
__global__ __launch_bounds__(256) void glue_swiglu_kernel(const bf16_t* __restrict__ a, int64_t lda, const bf16_t* __restrict__ u,
                                                          int64_t ldu, bf16_t* __restrict__ m, int64_t ldm, int64_t n, int64_t d) {
    const int64_t nvec = d / 8;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n * nvec) return;
    const int64_t row = idx / nvec, v = idx - row * nvec;
    float fa[8], fu[8];
    unpack8(*reinterpret_cast<const uint4*>(a + row * lda + v * 8), fa);
    unpack8(*reinterpret_cast<const uint4*>(u + row * ldu + v * 8), fu);
#pragma unroll
    for (int i = 0; i < 8; ++i) fa[i] = fa[i] / (1.f + __expf(-fa[i])) * fu[i];
    *reinterpret_cast<uint4*>(m + row * ldm + v * 8) = pack8(fa);
}

// h += delta (in place)
__global__ __launch_bounds__(256) void glue_add_kernel(bf16_t* __restrict__ h, int64_t ldh, const bf16_t* __restrict__ dl,
                                                       int64_t ldd, int64_t n, int64_t d) {
    const int64_t nvec = d / 8;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n * nvec) return;
    const int64_t row = idx / nvec, v = idx - row * nvec;
    float fh[8], fd[8];
    uint4* ph = reinterpret_cast<uint4*>(h + row * ldh + v * 8);
    unpack8(*ph, fh);
    unpack8(*reinterpret_cast<const uint4*>(dl + row * ldd + v * 8), fd);
#pragma unroll
    for (int i = 0; i < 8; ++i) fh[i] += fd[i];
    *ph = pack8(fh);
}

hipError_t launch_glue_rmsnorm(const bf16_t* x, int64_t ldx, bf16_t* y, int64_t ldy, const float* gain, int64_t n, int64_t d,
                               float eps, hipStream_t st) {
    if (n == 0 || d == 0) return hipSuccess;
    hipLaunchKernelGGL(glue_rmsnorm_kernel, dim3((unsigned)n), dim3(256), 0, st, x, ldx, y, ldy, gain, d, eps);
    return hipGetLastError();
}

hipError_t launch_glue_swiglu(const bf16_t* a, int64_t lda, const bf16_t* u, int64_t ldu, bf16_t* m, int64_t ldm, int64_t n,
                              int64_t d, hipStream_t st) {
    if (n == 0 || d == 0) return hipSuccess;
    const int64_t items = n * (d / 8);
    hipLaunchKernelGGL(glue_swiglu_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, st, a, lda, u, ldu, m, ldm, n, d);
    return hipGetLastError();
}

hipError_t launch_glue_add(bf16_t* h, int64_t ldh, const bf16_t* dl, int64_t ldd, int64_t n, int64_t d, hipStream_t st) {
    if (n == 0 || d == 0) return hipSuccess;
    const int64_t items = n * (d / 8);
    hipLaunchKernelGGL(glue_add_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, st, h, ldh, dl, ldd, n, d);
    return hipGetLastError();
}

}  // namespace agzo
