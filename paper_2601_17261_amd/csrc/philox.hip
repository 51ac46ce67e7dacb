// Standalone generator kernels: the Gaussian matrices of the method are functions of
// (seed, tag, row, col) only (Alg. 2: generated from a seed, regenerated at update time).
#include "agzo_internal.h"

namespace agzo {

__global__ __launch_bounds__(256) void philox_words_kernel(uint32_t* __restrict__ dst, int64_t rows, int cols,
                                                           int nquad, uint32_t s_lo, uint32_t s_hi, uint32_t tag) {
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t total = rows * nquad;
    if (idx >= total) return;
    int64_t row = idx / nquad;
    int quad = (int)(idx - row * nquad);
    uint4 x = philox4x32_10((uint32_t)row, (uint32_t)quad, tag, 0u, s_lo, s_hi);
    uint32_t v[4] = {x.x, x.y, x.z, x.w};
    int c0 = quad * 4;
    uint32_t* o = dst + row * cols + c0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
        if (c0 + i < cols) o[i] = v[i];
}

__global__ __launch_bounds__(256) void fill_normal_kernel(float* __restrict__ dst, int64_t rows, int cols, int nquad,
                                                          uint32_t s_lo, uint32_t s_hi, uint32_t tag, int vec_ok) {
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t total = rows * nquad;
    if (idx >= total) return;
    int64_t row = idx / nquad;
    int quad = (int)(idx - row * nquad);
    float4 z = philox_normal4(s_lo, s_hi, tag, (uint32_t)row, (uint32_t)quad);
    int c0 = quad * 4;
    float* o = dst + row * cols + c0;
    if (vec_ok) {
        *reinterpret_cast<float4*>(o) = z;
    } else {
        float v[4] = {z.x, z.y, z.z, z.w};
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (c0 + i < cols) o[i] = v[i];
    }
}

// Omega^T as three bf16 planes [3][rp][n_pad] (hi, mid, lo of each fp32 normal); columns >= r and
// tokens >= n are zero.  One thread makes one token's four columns.
__device__ __forceinline__ void fill_normal_packT_body(bf16_t* __restrict__ dst, int64_t n, int64_t n_pad, int r, int rp,
                                                       uint32_t s_lo, uint32_t s_hi, uint32_t tag, uint32_t bx, uint32_t by) {
    int64_t t = (int64_t)bx * 256 + threadIdx.x;
    int quad = (int)by;
    if (t >= n_pad) return;
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    if (t < n && quad * 4 < r) {
        float4 z = philox_normal4(s_lo, s_hi, tag, (uint32_t)t, (uint32_t)quad);
        v[0] = z.x; v[1] = z.y; v[2] = z.z; v[3] = z.w;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int k = quad * 4 + i;
        float f = (k < r) ? v[i] : 0.f;
        bf16_t hi, mid, lo;
        split3_bf16(f, hi, mid, lo);
        dst[((int64_t)0 * rp + k) * n_pad + t] = hi;
        dst[((int64_t)1 * rp + k) * n_pad + t] = mid;
        dst[((int64_t)2 * rp + k) * n_pad + t] = lo;
    }
}

__global__ __launch_bounds__(256) void fill_normal_packT_kernel(bf16_t* __restrict__ dst, int64_t n, int64_t n_pad,
                                                                int r, int rp, uint32_t s_lo, uint32_t s_hi,
                                                                uint32_t tag) {
    fill_normal_packT_body(dst, n, n_pad, r, rp, s_lo, s_hi, tag, blockIdx.x, blockIdx.y);
}

__global__ __launch_bounds__(256) void fill_normal_packT_many_kernel(const KBatch<FillPackTArgs> tb) {
    uint32_t bx, by;
    const FillPackTArgs& a = tb.a[kbatch_find(tb, bx, by)];
    fill_normal_packT_body(a.dst, a.n, a.n_pad, a.r, a.rp, (uint32_t)a.seed, (uint32_t)(a.seed >> 32), a.tag, bx, by);
}

hipError_t launch_philox_words(uint32_t* dst, int64_t rows, int cols, uint64_t seed, uint32_t tag, hipStream_t st) {
    if (rows == 0 || cols == 0) return hipSuccess;
    int nquad = (cols + 3) / 4;
    int64_t total = rows * nquad;
    dim3 grid((unsigned)((total + 255) / 256));
    hipLaunchKernelGGL(philox_words_kernel, grid, dim3(256), 0, st, dst, rows, cols, nquad, (uint32_t)seed,
                       (uint32_t)(seed >> 32), tag);
    return hipGetLastError();
}

hipError_t launch_fill_normal(float* dst, int64_t rows, int cols, uint64_t seed, uint32_t tag, hipStream_t st) {
    if (rows == 0 || cols == 0) return hipSuccess;
    int nquad = (cols + 3) / 4;
    int64_t total = rows * nquad;
    int vec_ok = (cols % 4 == 0) && ((reinterpret_cast<uintptr_t>(dst) & 15) == 0);
    dim3 grid((unsigned)((total + 255) / 256));
    hipLaunchKernelGGL(fill_normal_kernel, grid, dim3(256), 0, st, dst, rows, cols, nquad, (uint32_t)seed,
                       (uint32_t)(seed >> 32), tag, vec_ok);
    return hipGetLastError();
}

hipError_t launch_fill_normal_packT(bf16_t* dst, int64_t n, int64_t n_pad, int r, int rp, uint64_t seed, uint32_t tag,
                                    hipStream_t st) {
    if (n_pad == 0) return hipSuccess;
    dim3 grid((unsigned)((n_pad + 255) / 256), (unsigned)(rp / 4));
    hipLaunchKernelGGL(fill_normal_packT_kernel, grid, dim3(256), 0, st, dst, n, n_pad, r, rp, (uint32_t)seed,
                       (uint32_t)(seed >> 32), tag);
    return hipGetLastError();
}

hipError_t launch_fill_normal_packT_many(const FillPackTArgs* a, int n, hipStream_t st) {
    if (n < 0 || n > kBatchMax) return hipErrorInvalidValue;
    KBatch<FillPackTArgs> tb;
    tb.n = 0;
    uint64_t blocks = 0;
    for (int m = 0; m < n; ++m) {
        if (a[m].n_pad == 0) continue;
        const uint32_t gx = (uint32_t)((a[m].n_pad + 255) / 256);
        tb.first[tb.n] = (uint32_t)blocks;
        tb.gx[tb.n] = gx;
        tb.a[tb.n++] = a[m];
        blocks += (uint64_t)gx * (uint32_t)(a[m].rp / 4);
    }
    if (tb.n == 0) return hipSuccess;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(fill_normal_packT_many_kernel, dim3((unsigned)blocks), dim3(256), 0, st, tb);
    return hipGetLastError();
}

}  // namespace agzo
