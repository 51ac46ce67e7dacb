// Scalar tail of the step: final (fixed-order, fp64) loss sum and the two-point scalar of
// Eq. 10 / Alg. 2, g = (L+ - L-)/(2 eps) or, one-sided, (L+ - L0)/eps.  Everything stays on the
// device so a step never synchronises the host.
#include "agzo_internal.h"

namespace agzo {

__global__ __launch_bounds__(256) void finish_loss_kernel(const double* __restrict__ partials, int n, double scale,
                                                          double* __restrict__ out) {
    __shared__ double red[256];
    const int tid = threadIdx.x;
    double s = 0.0;
    partials += (int64_t)blockIdx.x * n;
    for (int i = tid; i < n; i += 256) s += partials[i];
    red[tid] = s;
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

hipError_t launch_finish_loss(const double* partials, int n, double scale, double* out, int nout, hipStream_t st) {
    hipLaunchKernelGGL(finish_loss_kernel, dim3(nout), dim3(256), 0, st, partials, n, scale, out);
    return hipGetLastError();
}

hipError_t launch_two_point(double* out4, float eps, int one_sided, hipStream_t st) {
    hipLaunchKernelGGL(two_point_kernel, dim3(1), dim3(64), 0, st, out4, eps, one_sided);
    return hipGetLastError();
}

}  // namespace agzo
