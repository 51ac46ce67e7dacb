// Scalar tail of the step: final (fixed-order, fp64) loss sum and the two-point scalar of
// Eq. 10 / Alg. 2, g = (L+ - L-)/(2 eps) or, one-sided, (L+ - L0)/eps.  Everything stays on the
// device so a step never synchronises the host.
#include "agzo_internal.h"

namespace agzo {

// this thread's share of sum(p[0..n)) for a 256-thread workgroup: four independent strided sums keep four loads in
// flight (the finishing kernels are one workgroup each, bound by latency); the order is fixed
__device__ __forceinline__ double strided_sum4(const double* __restrict__ p, int n, int tid) {
    double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
    int i = tid;
    for (; i + 768 < n; i += 1024) {
        s0 += p[i]; s1 += p[i + 256]; s2 += p[i + 512]; s3 += p[i + 768];
    }
    for (; i < n; i += 256) s0 += p[i];
    return (s0 + s1) + (s2 + s3);
}

__global__ __launch_bounds__(256) void finish_loss_kernel(const double* __restrict__ partials, int n, double scale,
                                                          double* __restrict__ out) {
    __shared__ double red[256];
    const int tid = threadIdx.x;
    red[tid] = strided_sum4(partials + (int64_t)blockIdx.x * n, n, tid);
    __syncthreads();
    for (int k = 128; k > 0; k >>= 1) {
        if (tid < k) red[tid] += red[tid + k];
        __syncthreads();
    }
    if (tid == 0) out[blockIdx.x] = red[0] * scale;
}

// out4 = {L0, L+, L-, g}
__global__ void two_point_kernel(double* __restrict__ out4, float eps, int one_sided) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        const double e = (double)eps;
        if (one_sided) {
            out4[2] = 0.0;   // L- is not evaluated in the one-sided form
            out4[3] = (out4[1] - out4[0]) / e;
        } else {
            out4[3] = (out4[1] - out4[2]) / (2.0 * e);
        }
    }
}

// finish_loss for nphase (2 or 3) consecutive partial arrays and two_point in one launch: out4 = {L0, L+, L-, g}.
// Same summation order per loss as finish_loss_kernel.
__global__ __launch_bounds__(256) void finish_two_point_kernel(const double* __restrict__ partials, int n, double scale,
                                                               int nphase, double* __restrict__ out4, float eps,
                                                               int one_sided) {
    __shared__ double red[256];
    __shared__ double loss[3];
    const int tid = threadIdx.x;
    for (int ph = 0; ph < nphase; ++ph) {
        red[tid] = strided_sum4(partials + (int64_t)ph * n, n, tid);
        __syncthreads();
        for (int k = 128; k > 0; k >>= 1) {
            if (tid < k) red[tid] += red[tid + k];
            __syncthreads();
        }
        if (tid == 0) loss[ph] = red[0] * scale;
        __syncthreads();
    }
    if (tid == 0) {
        const double e = (double)eps;
        out4[0] = loss[0];
        out4[1] = loss[1];
        if (one_sided) {
            out4[2] = 0.0;   // L- is not evaluated in the one-sided form
            out4[3] = (loss[1] - loss[0]) / e;
        } else {
            out4[2] = loss[2];
            out4[3] = (loss[1] - loss[2]) / (2.0 * e);
        }
    }
}

// ---- cross-entropy -----------------------------------------------------------------------------
// one thread per token: merge the chunk statistics, loss_t = log(sum exp) - logit[target]; block sums
// of (loss, count) go to scratch[2*block], the last stage divides.
__global__ __launch_bounds__(256) void ce_combine_kernel(const float2* __restrict__ ms, const float* __restrict__ tl,
                                                         const int32_t* __restrict__ target, int64_t M, int64_t N,
                                                         int nchunk, double* __restrict__ scratch) {
    __shared__ double rs[256], rc[256];
    const int tid = threadIdx.x;
    const int ph = blockIdx.y;
    const int64_t t = (int64_t)blockIdx.x * 256 + tid;
    double loss = 0.0, cnt = 0.0;
    if (t < M && target[t] >= 0 && target[t] < N) {   // an id outside the layer's outputs has no logit: skipped
        const float2* m = ms + (int64_t)ph * nchunk * M + t;
        float mx = -INFINITY;
        for (int c = 0; c < nchunk; ++c) mx = fmaxf(mx, m[(int64_t)c * M].x);
        double s = 0.0;
        for (int c = 0; c < nchunk; ++c) {
            const float2 v = m[(int64_t)c * M];
            s += (double)v.y * exp((double)v.x - (double)mx);
        }
        loss = log(s) + (double)mx - (double)tl[(int64_t)ph * M + t];
        cnt = 1.0;
    }
    rs[tid] = loss; rc[tid] = cnt;
    __syncthreads();
    for (int k = 128; k > 0; k >>= 1) {
        if (tid < k) { rs[tid] += rs[tid + k]; rc[tid] += rc[tid + k]; }
        __syncthreads();
    }
    if (tid == 0) {
        scratch[((int64_t)ph * gridDim.x + blockIdx.x) * 2] = rs[0];
        scratch[((int64_t)ph * gridDim.x + blockIdx.x) * 2 + 1] = rc[0];
    }
}

__global__ __launch_bounds__(256) void ce_finish_kernel(const double* __restrict__ scratch, int nblk, double* __restrict__ out) {
    __shared__ double rs[256], rc[256];
    const int tid = threadIdx.x, ph = blockIdx.x;
    double s = 0.0, c = 0.0;
    for (int i = tid; i < nblk; i += 256) {
        s += scratch[((int64_t)ph * nblk + i) * 2];
        c += scratch[((int64_t)ph * nblk + i) * 2 + 1];
    }
    rs[tid] = s; rc[tid] = c;
    __syncthreads();
    for (int k = 128; k > 0; k >>= 1) {
        if (tid < k) { rs[tid] += rs[tid + k]; rc[tid] += rc[tid + k]; }
        __syncthreads();
    }
    if (tid == 0) out[ph] = rc[0] > 0.0 ? rs[0] / rc[0] : 0.0;
}

hipError_t launch_ce_combine(const void* ms, const float* tl, const int32_t* target, int64_t M, int64_t N, int nchunk,
                             int nphase, double* scratch, double* out, hipStream_t st) {
    const int nblk = (int)((M + 255) / 256);
    hipLaunchKernelGGL(ce_combine_kernel, dim3(nblk, nphase), dim3(256), 0, st, reinterpret_cast<const float2*>(ms), tl,
                       target, M, N, nchunk, scratch);
    hipLaunchKernelGGL(ce_finish_kernel, dim3(nphase), dim3(256), 0, st, scratch, nblk, out);
    return hipGetLastError();
}

// fp32-storage path: one workgroup per token row of stored logits, fp64 statistics
__global__ __launch_bounds__(256) void ce_rows_f32_kernel(const float* __restrict__ Y, int64_t ldy, int64_t M, int64_t N,
                                                          const int32_t* __restrict__ target, double* __restrict__ scratch) {
    __shared__ double red[256];
    const int tid = threadIdx.x;
    const int64_t t = blockIdx.x;
    const int tgt = target[t];
    if (tgt < 0 || tgt >= N) {   // ignored row; an id outside the layer's outputs has no logit and is skipped too
        if (tid == 0) { scratch[t * 2] = 0.0; scratch[t * 2 + 1] = 0.0; }
        return;
    }
    const float* y = Y + t * ldy;
    double mx = -INFINITY;
    for (int64_t j = tid; j < N; j += 256) mx = fmax(mx, (double)y[j]);
    red[tid] = mx;
    __syncthreads();
    for (int k = 128; k > 0; k >>= 1) {
        if (tid < k) red[tid] = fmax(red[tid], red[tid + k]);
        __syncthreads();
    }
    mx = red[0];
    __syncthreads();
    double s = 0.0;
    for (int64_t j = tid; j < N; j += 256) s += exp((double)y[j] - mx);
    red[tid] = s;
    __syncthreads();
    for (int k = 128; k > 0; k >>= 1) {
        if (tid < k) red[tid] += red[tid + k];
        __syncthreads();
    }
    if (tid == 0) {
        scratch[t * 2] = log(red[0]) + mx - (double)y[tgt];
        scratch[t * 2 + 1] = 1.0;
    }
}

hipError_t launch_ce_rows_f32(const float* Y, int64_t ldy, int64_t M, int64_t N, const int32_t* target, double* scratch,
                              double* out, hipStream_t st) {
    hipLaunchKernelGGL(ce_rows_f32_kernel, dim3((unsigned)M), dim3(256), 0, st, Y, ldy, M, N, target, scratch);
    hipLaunchKernelGGL(ce_finish_kernel, dim3(1), dim3(256), 0, st, scratch, (int)M, out);
    return hipGetLastError();
}

hipError_t launch_finish_loss(const double* partials, int n, double scale, double* out, int nout, hipStream_t st) {
    hipLaunchKernelGGL(finish_loss_kernel, dim3(nout), dim3(256), 0, st, partials, n, scale, out);
    return hipGetLastError();
}

hipError_t launch_finish_two_point(const double* partials, int n, double scale, int nphase, double* out4, float eps,
                                   int one_sided, hipStream_t st) {
    hipLaunchKernelGGL(finish_two_point_kernel, dim3(1), dim3(256), 0, st, partials, n, scale, nphase, out4, eps, one_sided);
    return hipGetLastError();
}

hipError_t launch_two_point(double* out4, float eps, int one_sided, hipStream_t st) {
    hipLaunchKernelGGL(two_point_kernel, dim3(1), dim3(64), 0, st, out4, eps, one_sided);
    return hipGetLastError();
}

}  // namespace agzo
