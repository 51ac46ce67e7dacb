// Orthonormalisation steps of Alg. 1 ("[Q, ~] <- qr(Y)") for a tall d x r matrix, r <= 64:
// CholeskyQR2.  Gram matrix, Cholesky factor and triangular inverse are fp64; the first pass
// keeps its result in fp64 so the second pass starts from un-rounded data.  R from a Cholesky
// factor has a positive diagonal, which is the unique thin-QR factorisation of a full-rank Y.
// A non-positive pivot (rank-deficient sketch) raises a device flag instead of producing NaNs.
#include "agzo_internal.h"

namespace agzo {

constexpr int QR_ROWS = 64;    // rows per workgroup

static inline int64_t qr_blocks(int64_t d) { return (d + QR_ROWS - 1) / QR_ROWS; }

size_t qr_workspace_bytes(int64_t d, int r) {
    // [Q1 fp64 d*r][gram partials nblk*r*r fp64]
    return (size_t)d * r * sizeof(double) + (size_t)qr_blocks(d) * r * r * sizeof(double);
}

// partial[b][a][c] = sum over the block's rows of Y[i][a] * Y[i][c]
template <typename Tin>
__global__ __launch_bounds__(256) void gram_partial_kernel(const Tin* __restrict__ Y, int64_t d, int r,
                                                           double* __restrict__ partial) {
    extern __shared__ __align__(16) double qr_smem[];   // Ys[QR_ROWS][r + 1]
    double* Ys = qr_smem;
    const int ld = r + 1;
    const int tid = threadIdx.x;
    const int64_t i0 = (int64_t)blockIdx.x * QR_ROWS;
    const int rows = (int)min((int64_t)QR_ROWS, d - i0);
    for (int e = tid; e < rows * r; e += 256) Ys[(e / r) * ld + e % r] = (double)Y[i0 * r + e];
    __syncthreads();
    for (int e = tid; e < r * r; e += 256) {
        const int a = e / r, c = e % r;
        double s = 0.0;
        for (int i = 0; i < rows; ++i) s = fma(Ys[i * ld + a], Ys[i * ld + c], s);
        partial[(int64_t)blockIdx.x * r * r + e] = s;
    }
}

// every workgroup: G = sum of partials (fixed order); R = chol(G) upper; Rinv; then its rows: Q = Y Rinv
template <typename Tin, typename Tout>
__global__ __launch_bounds__(256) void chol_apply_kernel(const Tin* __restrict__ Y, int64_t d, int r,
                                                         const double* __restrict__ partial, int nblk,
                                                         Tout* __restrict__ Q, int* __restrict__ flag) {
    extern __shared__ __align__(16) double qr_smem[];   // G_(r, r+1) (becomes R, upper), RI_(r, r+1)
    const int ld = r + 1;
    double* Gm = qr_smem;
    double* Ri = qr_smem + r * ld;
    __shared__ int bad;
    const int tid = threadIdx.x;
#define G_(a, c) Gm[(a) * ld + (c)]
#define RI_(a, c) Ri[(a) * ld + (c)]
    if (tid == 0) bad = 0;
    for (int e = tid; e < r * r; e += 256) {
        double s = 0.0;
        for (int b = 0; b < nblk; ++b) s += partial[(int64_t)b * r * r + e];
        G_(e / r, e % r) = s;
    }
    __syncthreads();
    // right-looking Cholesky, upper factor: G = R^T R
    for (int j = 0; j < r; ++j) {
        if (tid == 0) {
            double piv = G_(j, j);
            if (!(piv > 0.0)) { bad = 1; piv = 1.0; }
            G_(j, j) = sqrt(piv);
        }
        __syncthreads();
        const double rjj = G_(j, j);
        for (int c = j + 1 + tid; c < r; c += 256) G_(j, c) /= rjj;
        __syncthreads();
        // trailing update: G_(a, c) -= R[j][a] * R[j][c] for j < a <= c
        const int n = r - j - 1;
        for (int e = tid; e < n * n; e += 256) {
            const int a = j + 1 + e / n, c = j + 1 + e % n;
            if (c >= a) G_(a, c) -= G_(j, a) * G_(j, c);
        }
        __syncthreads();
    }
    // inverse of the upper-triangular R, one column per thread (back substitution on e_c)
    if (tid < r) {
        const int c = tid;
        for (int i = c + 1; i < r; ++i) RI_(i, c) = 0.0;
        RI_(c, c) = 1.0 / G_(c, c);
        for (int i = c - 1; i >= 0; --i) {
            double s = 0.0;
            for (int k = i + 1; k <= c; ++k) s = fma(G_(i, k), RI_(k, c), s);
            RI_(i, c) = -s / G_(i, i);
        }
    }
    __syncthreads();
    if (bad && tid == 0 && blockIdx.x == 0) *flag = 1;
    const int64_t i0 = (int64_t)blockIdx.x * QR_ROWS;
    const int rows = (int)min((int64_t)QR_ROWS, d - i0);
    for (int e = tid; e < rows * r; e += 256) {
        const int i = e / r, c = e % r;
        const Tin* y = Y + (i0 + i) * r;
        double s = 0.0;
        for (int k = 0; k <= c; ++k) s = fma((double)y[k], RI_(k, c), s);
        Q[(i0 + i) * r + c] = (Tout)s;
    }
#undef G_
#undef RI_
}

hipError_t launch_qr(const float* S, int64_t d, int r, float* Q, void* workspace, int* numeric_flag, hipStream_t st) {
    if (d == 0) return hipSuccess;
    const int nblk = (int)qr_blocks(d);
    double* Q1 = reinterpret_cast<double*>(workspace);
    double* partial = Q1 + d * r;
    dim3 grid((unsigned)nblk), block(256);
    const size_t sm_gram = (size_t)QR_ROWS * (r + 1) * sizeof(double);
    const size_t sm_chol = (size_t)2 * r * (r + 1) * sizeof(double);
    static bool attr_set = false;
    if (!attr_set) {
        const int big = 2 * kMaxRank * (kMaxRank + 1) * (int)sizeof(double);
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(chol_apply_kernel<float, double>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, big);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(chol_apply_kernel<double, float>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, big);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(gram_partial_kernel<float>, grid, block, sm_gram, st, S, d, r, partial);
    hipLaunchKernelGGL((chol_apply_kernel<float, double>), grid, block, sm_chol, st, S, d, r, partial, nblk, Q1, numeric_flag);
    hipLaunchKernelGGL(gram_partial_kernel<double>, grid, block, sm_gram, st, Q1, d, r, partial);
    hipLaunchKernelGGL((chol_apply_kernel<double, float>), grid, block, sm_chol, st, Q1, d, r, partial, nblk, Q, numeric_flag);
    return hipGetLastError();
}

}  // namespace agzo
