// Orthonormalisation steps of Alg. 1 ("[Q, ~] <- qr(Y)") for a tall d x r matrix, r <= 64:
// CholeskyQR2, everything past the fp32 input in fp64.  R from a Cholesky factor has a positive
// diagonal, which is the unique thin-QR factorisation of a full-rank Y.  A non-positive pivot
// (rank-deficient sketch) raises a device flag instead of producing NaNs.
//
// Three launches per QR, coherence between them by kernel boundaries only (no device-scope fences):
//   1. gram        : Gram partials of Y per 128-row block (v_mfma_f64_16x16x4_f64)
//   2. apply_gram  : every block sums the partials in block order and one of its waves factors the
//                    r x r matrix in registers (lane = column, rows broadcast with v_readlane) -> R1;
//                    Q1 = Y R1^-1 by forward substitution, one thread per row (fp64, stored), then
//                    the Gram partials of Q1
//   3. apply_final : the same reduction and factorisation -> R2; Q = Q1 R2^-1 (fp32), optionally
//                    also as three bf16 planes [3][rp][d]
// The orthonormalisations between power steps run a single pass (launches 1 and 3 only, launch 3 applying R1 to Y):
// Q1 = Q R2 with R2 upper triangular and positive on the diagonal, so the next sketch X^T X Q1 = (X^T X Q) R2 has
// the same thin-QR Q factor; the second pass only matters for the orthonormality of the basis that is returned.
// When the input arrives as per-token-range partial sketches, launch 1 sums them (fp64, fixed order)
// on the way in and stores the fp32 sketch, so no separate reduction kernel is needed.
#include "agzo_internal.h"

namespace agzo {

typedef double doublex4 __attribute__((ext_vector_type(4)));

constexpr int QR_ROWS = 128;   // rows per workgroup

static inline int64_t qr_blocks(int64_t d) { return (d + QR_ROWS - 1) / QR_ROWS; }

size_t qr_workspace_bytes(int64_t d, int r) {
    const int rp = (r + 15) / 16 * 16;
    // [Q1 fp64 d*r][gram partials of Y and of Q1: nblk*rp*rp fp64 each]
    return (size_t)d * r * sizeof(double) + (size_t)2 * qr_blocks(d) * rp * rp * sizeof(double);
}

__device__ __forceinline__ double readlane_f64(double v, int lane) {
    const uint64_t u = __double_as_longlong(v);
    const uint32_t lo = __builtin_amdgcn_readlane((int)(uint32_t)u, lane);
    const uint32_t hi = __builtin_amdgcn_readlane((int)(uint32_t)(u >> 32), lane);
    return __longlong_as_double(((uint64_t)hi << 32) | lo);
}

// One wave factors G (RP x RP, row-major fp64 in LDS, leading dimension RP) = R^T R in registers:
// lane c owns column c.  On exit G's upper triangle holds R, its diagonal 1 / R[j][j] (what the
// substitution needs).  Padding columns (>= r) carry a unit diagonal.  Returns nonzero on a bad pivot.
template <int RP>
__device__ int chol_wave(double* G, int r) {
    const int lane = threadIdx.x & 63;
    const int c = lane < RP ? lane : RP - 1;
    double col[RP];
#pragma unroll
    for (int a = 0; a < RP; ++a) col[a] = G[a * RP + c];
    int bad = 0;
#pragma unroll
    for (int j = 0; j < RP; ++j) {
        double piv = readlane_f64(col[j], j);
        if (j >= r) piv = 1.0;
        if (!(piv > 0.0)) { bad = 1; piv = 1.0; }
        // 1/sqrt(piv): hardware estimate refined by two Newton steps (full fp64 accuracy, no divide)
        double inv = __builtin_amdgcn_rsq(piv);
        inv = inv * fma(-0.5 * piv * inv, inv, 1.5);
        inv = inv * fma(-0.5 * piv * inv, inv, 1.5);
        const double rowj = col[j] * inv;                 // lane c: R[j][c]
        col[j] = (lane == j) ? inv : rowj;                // keep 1/R[j][j] on the diagonal
#pragma unroll
        for (int a = j + 1; a < RP; ++a) col[a] = fma(-readlane_f64(rowj, a), rowj, col[a]);
    }
    if (lane < RP) {
#pragma unroll
        for (int a = 0; a < RP; ++a) G[a * RP + lane] = col[a];
    }
    return bad;
}

__device__ int chol_dispatch(double* G, int r, int rp) {
    switch (rp) {
        case 16: return chol_wave<16>(G, r);
        case 32: return chol_wave<32>(G, r);
        case 48: return chol_wave<48>(G, r);
        default: return chol_wave<64>(G, r);
    }
}

// Gram partial of the block's rows (fp64 in LDS: Ys[row][ld], zero padded to a multiple of 4 rows and rp
// columns) with the fp64 matrix cores, written to partial[blockIdx.x][rp][rp].
__device__ void gram_partial(const double* Ys, int ld, int rows_pad, int rp, double* partial) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nb = rp / 16;
    // block pair (bi, bj) of the Gram matrix per wave, round robin; operand lane layout of the 16x16x4
    // fp64 MFMA: lane l supplies element (l % 16, k = l / 16) of both A (rows = Gram row) and B
    for (int blk = wave; blk < nb * nb; blk += 4) {
        const int bi = blk / nb, bj = blk % nb;
        doublex4 acc = {0.0, 0.0, 0.0, 0.0};
        for (int k0 = 0; k0 < rows_pad; k0 += 4) {
            const double a = Ys[(k0 + (lane >> 4)) * ld + bi * 16 + (lane & 15)];
            const double b = Ys[(k0 + (lane >> 4)) * ld + bj * 16 + (lane & 15)];
            acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc, 0, 0, 0);
        }
        // D (measured on gfx950): register i of lane l is row 4*i + l/16, column l % 16
#pragma unroll
        for (int i = 0; i < 4; ++i)
            partial[((int64_t)blockIdx.x * rp + bi * 16 + 4 * i + (lane >> 4)) * rp + bj * 16 + (lane & 15)] = acc[i];
    }
}

// Every block: Gs <- sum over blocks of partial (block order, sixteen loads in flight), then wave 0
// factors it in place (upper factor, reciprocal diagonal).  Block 0 reports a bad pivot.
__device__ void reduce_and_factor(const double* partial, int nblk, double* Gs, int r, int rp, int* flag) {
    const int tid = threadIdx.x;
    for (int e = tid; e < rp * rp; e += blockDim.x) {
        double a16[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) a16[u] = 0.0;
        for (int b0 = 0; b0 < nblk; b0 += 16) {
#pragma unroll
            for (int u = 0; u < 16; ++u)
                if (b0 + u < nblk) a16[u] += partial[(int64_t)(b0 + u) * rp * rp + e];
        }
#pragma unroll
        for (int s = 8; s > 0; s >>= 1)
#pragma unroll
            for (int u = 0; u < s; ++u) a16[u] += a16[u + s];
        Gs[e] = a16[0];
    }
    __syncthreads();
    if (tid < 64) {
        const int bad = chol_dispatch(Gs, r, rp);
        if (bad && tid == 0 && blockIdx.x == 0) *flag = 1;
    }
    __syncthreads();
}

// row <- row R^-1 for upper-triangular R held in LDS with reciprocal diagonal (forward substitution);
// the row stays in registers, R is read with broadcast loads
template <int RP, typename Tin>
__device__ __forceinline__ void solve_row_t(const Tin* y, const double* Rl, int r, double* q_out) {
    double q[RP];
#pragma unroll
    for (int c = 0; c < RP; ++c) {
        double s = (c < r) ? (double)y[c] : 0.0;
#pragma unroll
        for (int k = 0; k < c; ++k) s = fma(-q[k], Rl[k * RP + c], s);
        q[c] = s * Rl[c * RP + c];
    }
#pragma unroll
    for (int c = 0; c < RP; ++c) q_out[c] = q[c];
}

template <typename Tin>
__device__ __forceinline__ void solve_row(const Tin* y, const double* Rl, int r, int rp, double* q) {
    switch (rp) {
        case 16: solve_row_t<16>(y, Rl, r, q); break;
        case 32: solve_row_t<32>(y, Rl, r, q); break;
        case 48: solve_row_t<48>(y, Rl, r, q); break;
        default: solve_row_t<64>(y, Rl, r, q); break;
    }
}

// launch 1.  Input: S fp32 [d][r], or (splits != nullptr) partial sketches [nsplit][d][rp] whose sum is
// stored to S_out as fp32 and used (in its rounded form) for the factorisation.
__global__ __launch_bounds__(256) void qr_gram_kernel(const float* __restrict__ S, const float* __restrict__ splits,
                                                      int nsplit, float* __restrict__ S_out, int64_t d, int r, int rp,
                                                      double* __restrict__ partial) {
    extern __shared__ __align__(16) double qr_smem[];
    const int ld = rp + 1;
    double* Ys = qr_smem;                 // [QR_ROWS][ld]
    const int tid = threadIdx.x;
    const int64_t i0 = (int64_t)blockIdx.x * QR_ROWS;
    const int rows = (int)min((int64_t)QR_ROWS, d - i0);
    const int rows_pad = (rows + 3) & ~3;
    if (splits != nullptr) {
        // sum of the partial sketches: 8 elements per thread and 4 splits per round, 32 loads in flight
        for (int base = 0; base < rows_pad * rp; base += 256 * 8) {
            double acc[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) acc[u] = 0.0;
            for (int sp0 = 0; sp0 < nsplit; sp0 += 4) {
                float v[4][8];
#pragma unroll
                for (int s4 = 0; s4 < 4; ++s4)
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int e = base + u * 256 + tid;
                        const int i = e / rp, k = e % rp;
                        const bool ok = (e < rows_pad * rp) && (i < rows) && (sp0 + s4 < nsplit);
                        v[s4][u] = ok ? splits[((int64_t)(sp0 + s4) * d + i0 + i) * rp + k] : 0.f;
                    }
#pragma unroll
                for (int s4 = 0; s4 < 4; ++s4)
#pragma unroll
                    for (int u = 0; u < 8; ++u) acc[u] += (double)v[s4][u];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int e = base + u * 256 + tid;
                if (e >= rows_pad * rp) continue;
                const int i = e / rp, k = e % rp;
                float f = 0.f;
                if (i < rows && k < r) {
                    f = (float)acc[u];
                    S_out[(i0 + i) * r + k] = f;
                }
                Ys[i * ld + k] = (double)f;
            }
        }
    } else {
        for (int e = tid; e < rows_pad * rp; e += 256) {
            const int i = e / rp, k = e % rp;
            const float v = (i < rows && k < r) ? S[(i0 + i) * r + k] : 0.f;
            Ys[i * ld + k] = (double)v;
        }
    }
    __syncthreads();
    gram_partial(Ys, ld, rows_pad, rp, partial);
}

// launch 2: R1 from the partials, Q1 = S R1^-1 for the block's rows (fp64, stored), Gram partials of Q1.
__global__ __launch_bounds__(256) void qr_apply_gram_kernel(const float* __restrict__ S, int64_t d, int r, int rp,
                                                            const double* __restrict__ partial1, int nblk,
                                                            double* __restrict__ Q1, double* __restrict__ partial2,
                                                            int* flag) {
    extern __shared__ __align__(16) double qr_smem[];
    const int ld = rp + 1;
    double* Ys = qr_smem;
    double* Gs = qr_smem + QR_ROWS * ld;
    const int tid = threadIdx.x;
    const int64_t i0 = (int64_t)blockIdx.x * QR_ROWS;
    const int rows = (int)min((int64_t)QR_ROWS, d - i0);
    const int rows_pad = (rows + 3) & ~3;
    for (int e = tid; e < rows_pad * ld; e += 256) Ys[e] = 0.0;
    reduce_and_factor(partial1, nblk, Gs, r, rp, flag);
    if (tid < rows) {
        double* q = Ys + tid * ld;
        solve_row(S + (i0 + tid) * r, Gs, r, rp, q);
        for (int c = 0; c < r; ++c) Q1[(i0 + tid) * r + c] = q[c];
    }
    __syncthreads();
    gram_partial(Ys, ld, rows_pad, rp, partial2);
}

// launch 3: Q = Q1 R2^-1, rounded to fp32; planes (nullable) receive the hi/mid/lo bf16 parts [3][rp][d].
// With Tin = float the same kernel closes a single-pass factorisation: Q = Y R1^-1 straight from launch 1's partials.
template <typename Tin>
__global__ __launch_bounds__(256) void qr_apply_final_kernel(const Tin* __restrict__ Q1, int64_t d, int r, int rp,
                                                             const double* __restrict__ partial2, int nblk,
                                                             float* __restrict__ Q, bf16_t* __restrict__ planes,
                                                             int* flag) {
    extern __shared__ __align__(16) double qr_smem[];
    const int ld = rp + 1;
    double* Gs = qr_smem;                 // [rp][rp]
    double* Qs = qr_smem + rp * rp;       // [QR_ROWS][ld]
    const int tid = threadIdx.x;
    const int64_t i0 = (int64_t)blockIdx.x * QR_ROWS;
    const int rows = (int)min((int64_t)QR_ROWS, d - i0);
    reduce_and_factor(partial2, nblk, Gs, r, rp, flag);
    if (tid < rows) {
        double* q = Qs + tid * ld;
        solve_row(Q1 + (i0 + tid) * r, Gs, r, rp, q);
        for (int c = 0; c < r; ++c) Q[(i0 + tid) * r + c] = (float)q[c];
        for (int c = r; c < rp; ++c) q[c] = 0.0;
    }
    if (planes == nullptr) return;
    __syncthreads();
    // row index fastest so that the plane stores (row-contiguous per k) coalesce
    for (int e = tid; e < QR_ROWS * rp; e += 256) {
        const int i = e % QR_ROWS, c = e / QR_ROWS;
        if (i >= rows) continue;
        bf16_t hi, mid, lo;
        split3_bf16((float)Qs[i * ld + c], hi, mid, lo);
        planes[((int64_t)0 * rp + c) * d + i0 + i] = hi;
        planes[((int64_t)1 * rp + c) * d + i0 + i] = mid;
        planes[((int64_t)2 * rp + c) * d + i0 + i] = lo;
    }
}

hipError_t launch_qr(const float* S, const float* splits, int nsplit, int rp, float* S_out, int64_t d, int r, float* Q,
                     bf16_t* planes, void* workspace, int* numeric_flag, bool refine, hipStream_t st) {
    if (d == 0) return hipSuccess;
    const int nblk = (int)qr_blocks(d);
    double* Q1 = reinterpret_cast<double*>(workspace);
    double* partial1 = Q1 + d * r;
    double* partial2 = partial1 + (size_t)nblk * rp * rp;
    dim3 grid((unsigned)nblk), block(256);
    const size_t sm_full = ((size_t)QR_ROWS * (rp + 1) + (size_t)rp * rp) * sizeof(double);
    static bool attr_set = false;
    if (!attr_set) {
        const int big = (QR_ROWS * (kMaxRank + 1) + kMaxRank * kMaxRank) * (int)sizeof(double);
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(qr_gram_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, big);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(qr_apply_gram_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, big);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(qr_apply_final_kernel<double>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, big);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(qr_apply_final_kernel<float>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, big);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const float* Sin = splits ? S_out : S;
    hipLaunchKernelGGL(qr_gram_kernel, grid, block, sm_full, st, S, splits, nsplit, S_out, d, r, rp, partial1);
    if (!refine) {
        hipLaunchKernelGGL(qr_apply_final_kernel<float>, grid, block, sm_full, st, Sin, d, r, rp, partial1, nblk, Q, planes,
                           numeric_flag);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(qr_apply_gram_kernel, grid, block, sm_full, st, Sin, d, r, rp, partial1, nblk, Q1, partial2,
                       numeric_flag);
    hipLaunchKernelGGL(qr_apply_final_kernel<double>, grid, block, sm_full, st, Q1, d, r, rp, partial2, nblk, Q, planes,
                       numeric_flag);
    return hipGetLastError();
}

}  // namespace agzo
