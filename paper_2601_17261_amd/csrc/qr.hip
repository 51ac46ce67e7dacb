// Orthonormalisation steps of Alg. 1 ("[Q, ~] <- qr(Y)") for a tall d x r matrix, r <= 64:
// CholeskyQR2, everything past the fp32 input in fp64.  R from a Cholesky factor has a positive
// diagonal, which is the unique thin-QR factorisation of a full-rank Y.  A non-positive pivot
// (rank-deficient sketch) raises a device flag instead of producing NaNs.
//
// Three launches per QR:
//   1. gram_chol      : Gram partials of Y per 128-row block (v_mfma_f64_16x16x4_f64); the block that
//                       finishes last sums them in block order and one wave factors the r x r matrix
//                       in registers (lane = column, rows broadcast with v_readlane)  -> R1
//   2. apply_gram_chol: Q1 = Y R1^-1 by forward substitution, one thread per row (fp64, stored), then
//                       Gram partials of Q1 and the last block's factorisation       -> R2
//   3. apply_final    : Q = Q1 R2^-1 (fp32), optionally also as three bf16 planes [3][rp][d]
// When the input arrives as per-token-range partial sketches, launch 1 sums them (fp64, fixed order)
// on the way in and stores the fp32 sketch, so no separate reduction kernel is needed.
#include "agzo_internal.h"

namespace agzo {

typedef double doublex4 __attribute__((ext_vector_type(4)));

constexpr int QR_ROWS = 128;   // rows per workgroup

static inline int64_t qr_blocks(int64_t d) { return (d + QR_ROWS - 1) / QR_ROWS; }

size_t qr_workspace_bytes(int64_t d, int r) {
    const int rp = (r + 15) / 16 * 16;
    // [Q1 fp64 d*r][gram partials nblk*rp*rp fp64][R1, R2: rp*rp fp64 each]
    return (size_t)d * r * sizeof(double) + (size_t)qr_blocks(d) * rp * rp * sizeof(double) +
           (size_t)2 * rp * rp * sizeof(double);
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
        const double inv = 1.0 / sqrt(piv);
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
// columns) with the fp64 matrix cores, written to `partial`; the last block to arrive reduces all
// partials in block order, factors, and stores the factor to Rout.  Gs: [rp][rp] LDS work matrix.
__device__ void gram_then_last_block_chol(const double* Ys, int ld, double* Gs, int rows_pad, int r, int rp, double* partial,
                                          int nblk, double* Rout, unsigned int* counter, int* flag) {
    __shared__ int is_last;
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
    __threadfence();                       // partials visible device-wide before the ticket is taken
    __syncthreads();
    if (tid == 0) {
        const unsigned int ticket = atomicAdd(counter, 1u);
        is_last = (ticket == (unsigned int)(nblk - 1));
    }
    __syncthreads();
    if (!is_last) return;
    __threadfence();                       // see every other block's partials
    for (int e = tid; e < rp * rp; e += blockDim.x) {
        // sixteen independent running sums so that the loads overlap; the order is fixed all the same
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
    if (wave == 0) {
        const int bad = chol_dispatch(Gs, r, rp);
        if (lane == 0) {
            if (bad) *flag = 1;
            *counter = 0u;                 // ready for the next launch on this stream
        }
    }
    __syncthreads();
    for (int e = tid; e < rp * rp; e += blockDim.x) Rout[e] = Gs[e];
}

// row <- row R^-1 for upper-triangular R held in LDS with reciprocal diagonal (forward substitution)
// q is the thread's own row in LDS (rows are an odd number of doubles apart: no bank conflicts)
template <typename Tin>
__device__ __forceinline__ void solve_row(const Tin* y, const double* Rl, int r, int rp, double* q) {
    for (int c = 0; c < r; ++c) {
        double s = (double)y[c];
        for (int k = 0; k < c; ++k) s = fma(-q[k], Rl[k * rp + c], s);
        q[c] = s * Rl[c * rp + c];
    }
}

// launch 1.  Input: S fp32 [d][r], or (splits != nullptr) partial sketches [nsplit][d][rp] whose sum is
// stored to S_out as fp32 and used (in its rounded form) for the factorisation.
__global__ __launch_bounds__(256) void qr_gram_chol_kernel(const float* __restrict__ S, const float* __restrict__ splits,
                                                           int nsplit, float* __restrict__ S_out, int64_t d, int r,
                                                           int rp, double* __restrict__ partial, int nblk,
                                                           double* __restrict__ R1, unsigned int* counter, int* flag) {
    extern __shared__ __align__(16) double qr_smem[];
    const int ld = rp + 1;
    double* Ys = qr_smem;                 // [QR_ROWS][ld]
    double* Gs = qr_smem + QR_ROWS * ld;  // [rp][rp]
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
    gram_then_last_block_chol(Ys, ld, Gs, rows_pad, r, rp, partial, nblk, R1, counter, flag);
}

// launch 2: Q1 = S R1^-1 for the block's rows (fp64, stored), then the Gram of Q1 as in launch 1.
__global__ __launch_bounds__(256) void qr_apply_gram_chol_kernel(const float* __restrict__ S, int64_t d, int r, int rp,
                                                                 const double* __restrict__ R1, double* __restrict__ Q1,
                                                                 double* __restrict__ partial, int nblk,
                                                                 double* __restrict__ R2, unsigned int* counter,
                                                                 int* flag) {
    extern __shared__ __align__(16) double qr_smem[];
    const int ld = rp + 1;
    double* Ys = qr_smem;
    double* Gs = qr_smem + QR_ROWS * ld;
    const int tid = threadIdx.x;
    const int64_t i0 = (int64_t)blockIdx.x * QR_ROWS;
    const int rows = (int)min((int64_t)QR_ROWS, d - i0);
    const int rows_pad = (rows + 3) & ~3;
    for (int e = tid; e < rp * rp; e += 256) Gs[e] = R1[e];
    for (int e = tid; e < rows_pad * ld; e += 256) Ys[e] = 0.0;
    __syncthreads();
    if (tid < rows) {
        double* q = Ys + tid * ld;
        solve_row(S + (i0 + tid) * r, Gs, r, rp, q);
        for (int c = 0; c < r; ++c) Q1[(i0 + tid) * r + c] = q[c];
    }
    __syncthreads();
    gram_then_last_block_chol(Ys, ld, Gs, rows_pad, r, rp, partial, nblk, R2, counter, flag);
}

// launch 3: Q = Q1 R2^-1, rounded to fp32; planes (nullable) receive the hi/mid/lo bf16 parts [3][rp][d]
__global__ __launch_bounds__(256) void qr_apply_final_kernel(const double* __restrict__ Q1, int64_t d, int r, int rp,
                                                             const double* __restrict__ R2, float* __restrict__ Q,
                                                             bf16_t* __restrict__ planes) {
    extern __shared__ __align__(16) double qr_smem[];
    const int ld = rp + 1;
    double* Gs = qr_smem;                 // [rp][rp]
    double* Qs = qr_smem + rp * rp;       // [QR_ROWS][ld]
    const int tid = threadIdx.x;
    const int64_t i0 = (int64_t)blockIdx.x * QR_ROWS;
    const int rows = (int)min((int64_t)QR_ROWS, d - i0);
    for (int e = tid; e < rp * rp; e += 256) Gs[e] = R2[e];
    __syncthreads();
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
                     bf16_t* planes, void* workspace, unsigned int* counter, int* numeric_flag, hipStream_t st) {
    if (d == 0) return hipSuccess;
    const int nblk = (int)qr_blocks(d);
    double* Q1 = reinterpret_cast<double*>(workspace);
    double* partial = Q1 + d * r;
    double* R1 = partial + (size_t)nblk * rp * rp;
    double* R2 = R1 + rp * rp;
    dim3 grid((unsigned)nblk), block(256);
    const size_t sm_full = ((size_t)QR_ROWS * (rp + 1) + (size_t)rp * rp) * sizeof(double);
    const size_t sm_apply = sm_full;
    static bool attr_set = false;
    if (!attr_set) {
        const int big = (QR_ROWS * (kMaxRank + 1) + kMaxRank * kMaxRank) * (int)sizeof(double);
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(qr_gram_chol_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, big);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(qr_apply_gram_chol_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, big);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(qr_apply_final_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, big);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const float* Sin = splits ? S_out : S;
    hipLaunchKernelGGL(qr_gram_chol_kernel, grid, block, sm_full, st, S, splits, nsplit, S_out, d, r, rp, partial, nblk, R1,
                       counter, numeric_flag);
    hipLaunchKernelGGL(qr_apply_gram_chol_kernel, grid, block, sm_full, st, Sin, d, r, rp, R1, Q1, partial, nblk, R2,
                       counter, numeric_flag);
    hipLaunchKernelGGL(qr_apply_final_kernel, grid, block, sm_apply, st, Q1, d, r, rp, R2, Q, planes);
    return hipGetLastError();
}

}  // namespace agzo
