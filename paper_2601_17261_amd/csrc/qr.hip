// Orthonormalisation steps of Alg. 1 ("[Q, ~] <- qr(Y)") for a tall d x r matrix, r <= 64:
// CholeskyQR2, everything past the fp32 input in fp64.  R from a Cholesky factor has a positive
// diagonal, which is the unique thin-QR factorisation of a full-rank Y.  A non-positive pivot
// (rank-deficient sketch) raises a device flag instead of producing NaNs.
//
// Three launches per QR, coherence between them by kernel boundaries only (no device-scope fences):
//   1. gram        : Gram partials of Y per 128-row block (v_mfma_f64_16x16x4_f64)
//   2. apply_gram  : every block sums the partials in block order and factors the r x r matrix in LDS
//                    (right-looking, the whole workgroup on the trailing update) -> R1;
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

// The workgroup factors G (rp x rp, row-major fp64 in LDS) = R^T R in place, right-looking, two barriers per column:
// on exit G's upper triangle holds R and its diagonal 1 / R[j][j] (what the substitution needs).  Padding columns
// (>= r) carry a unit diagonal.  Returns nonzero on a non-positive pivot (the same value in every thread).
__device__ int chol_block(double* G, int r, int rp) {
    __shared__ double dinv[kMaxRank];
    const int tid = threadIdx.x, nt = blockDim.x;
    int bad = 0;
    if (tid >= r && tid < rp) dinv[tid] = 1.0;            // padding columns: zero rows and columns, unit diagonal
    for (int j = 0; j < r; ++j) {                         // (they need no elimination step)
        __syncthreads();                                  // the trailing update of the previous column is complete
        double piv = G[j * rp + j];
        if (!(piv > 0.0)) { bad = 1; piv = 1.0; }
        // 1/sqrt(piv): hardware estimate refined by two Newton steps (full fp64 accuracy, no divide)
        double inv = __builtin_amdgcn_rsq(piv);
        inv = inv * fma(-0.5 * piv * inv, inv, 1.5);
        inv = inv * fma(-0.5 * piv * inv, inv, 1.5);
        if (tid == j) dinv[j] = inv;
        if (tid > j && tid < rp) G[j * rp + tid] *= inv;  // row j of R (the pivot itself stays in place until the end)
        __syncthreads();
        // trailing update of the upper triangle: G[a][c] -= R[j][a] R[j][c], j < a <= c
        const int m = rp - j - 1;
        for (int e = tid; e < m * m; e += nt) {
            const int a = j + 1 + e / m, c = j + 1 + e % m;
            if (c >= a) G[a * rp + c] = fma(-G[j * rp + a], G[j * rp + c], G[a * rp + c]);
        }
    }
    __syncthreads();
    if (tid < rp) G[tid * rp + tid] = dinv[tid];
    __syncthreads();
    return bad;
}

// Gram partial of the block's rows (fp64 in LDS: Ys[row][ld], zero padded to a multiple of 4 rows and rp
// columns) with the fp64 matrix cores, written to partial[blockIdx.x][rp][rp].
__device__ void gram_partial(const double* Ys, int ld, int rows_pad, int rp, double* partial, uint32_t bx) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nb = rp / 16;
    // operand lane layout of the 16x16x4 fp64 MFMA: lane l supplies element (l % 16, k = l / 16) of both A (rows =
    // Gram row) and B; D (measured on gfx950): register i of lane l is row 4*i + l/16, column l % 16
    if (nb == 1) {
        // a single 16 x 16 block: the four waves split the rows (a lone wave would walk all of them through a chain
        // of dependent MFMAs) and their sums are added in wave order
        __shared__ double quarter[4][256];
        const int chunk = ((rows_pad / 4 + 3) / 4) * 4;               // rows per wave, a multiple of 4
        const int k_begin = min(wave * chunk, rows_pad), k_end = min(k_begin + chunk, rows_pad);
        doublex4 acc = {0.0, 0.0, 0.0, 0.0};
        for (int k0 = k_begin; k0 < k_end; k0 += 4) {
            const double a = Ys[(k0 + (lane >> 4)) * ld + (lane & 15)];
            acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a, a, acc, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) quarter[wave][(4 * i + (lane >> 4)) * 16 + (lane & 15)] = acc[i];
        __syncthreads();
        partial[(int64_t)bx * 256 + tid] = (quarter[0][tid] + quarter[1][tid]) + (quarter[2][tid] + quarter[3][tid]);
        return;
    }
    // block pair (bi, bj) of the Gram matrix per wave, round robin
    for (int blk = wave; blk < nb * nb; blk += 4) {
        const int bi = blk / nb, bj = blk % nb;
        doublex4 acc = {0.0, 0.0, 0.0, 0.0};
        for (int k0 = 0; k0 < rows_pad; k0 += 4) {
            const double a = Ys[(k0 + (lane >> 4)) * ld + bi * 16 + (lane & 15)];
            const double b = Ys[(k0 + (lane >> 4)) * ld + bj * 16 + (lane & 15)];
            acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
            partial[((int64_t)bx * rp + bi * 16 + 4 * i + (lane >> 4)) * rp + bj * 16 + (lane & 15)] = acc[i];
    }
}

// Every block: Gs <- sum over blocks of partial (block order, up to 32 loads in flight), then the workgroup factors
// it in place (upper factor, reciprocal diagonal).  Block 0 reports a bad pivot.
__device__ void reduce_and_factor(const double* partial, int nblk, double* Gs, int r, int rp, int* flag, uint32_t bx) {
    const int tid = threadIdx.x;
    for (int e = tid; e < rp * rp; e += blockDim.x) {
        double sum = 0.0;
        for (int b0 = 0; b0 < nblk; b0 += 32) {
            double v[32];
#pragma unroll
            for (int u = 0; u < 32; ++u) v[u] = (b0 + u < nblk) ? partial[(int64_t)(b0 + u) * rp * rp + e] : 0.0;
#pragma unroll
            for (int u = 0; u < 32; ++u) sum += v[u];
        }
        Gs[e] = sum;
    }
    __syncthreads();
    const int bad = chol_block(Gs, r, rp);
    if (bad && tid == 0 && bx == 0) *flag = 1;
}

// the block's input row of this thread, requested before the reduction and factorisation so that its memory latency
// runs under them (RP is a compile-time bound, so the row lives in registers)
template <int RP, typename Tin>
__device__ __forceinline__ void load_row_t(const Tin* y, int r, bool active, Tin (&v)[RP]) {
#pragma unroll
    for (int c = 0; c < RP; ++c) v[c] = (active && c < r) ? y[c] : (Tin)0;
}

// row <- row R^-1 for upper-triangular R held in LDS with reciprocal diagonal (forward substitution);
// the row stays in registers, R is read with broadcast loads
template <int RP, typename Tin>
__device__ __forceinline__ void solve_row_t(const Tin (&y)[RP], const double* Rl, double* q_out) {
    double q[RP];
#pragma unroll
    for (int c = 0; c < RP; ++c) {
        double s = (double)y[c];
#pragma unroll
        for (int k = 0; k < c; ++k) s = fma(-q[k], Rl[k * RP + c], s);
        q[c] = s * Rl[c * RP + c];
    }
#pragma unroll
    for (int c = 0; c < RP; ++c) q_out[c] = q[c];
}

// launch 1.  Input: S fp32 [d][r], or (splits != nullptr) partial sketches [nsplit][d][rp] whose sum is
// stored to S_out as fp32 and used (in its rounded form) for the factorisation.
__device__ __forceinline__ void qr_gram_body(const float* __restrict__ S, const float* __restrict__ splits, int nsplit,
                                             float* __restrict__ S_out, int64_t d, int r, int rp,
                                             double* __restrict__ partial, uint32_t bx) {
    extern __shared__ __align__(16) double qr_smem[];
    const int ld = rp + 1;
    double* Ys = qr_smem;                 // [QR_ROWS][ld]
    const int tid = threadIdx.x;
    const int64_t i0 = (int64_t)bx * QR_ROWS;
    const int rows = (int)min((int64_t)QR_ROWS, d - i0);
    const int rows_pad = (rows + 3) & ~3;
    if (splits != nullptr) {
        // sum of the partial sketches: a block's rows are one contiguous run of rows * rp floats in every split, so the
        // loads are plain 16-byte vectors, all splits of a vector in flight together (fp64 sum in split order)
        const int nvec = rows * rp / 4, total_vec = rows_pad * rp / 4;
        const float* base = splits + i0 * rp;
        auto finish = [&](int v, const double (&acc)[4]) {
            const int i = (v * 4) / rp, k0 = (v * 4) % rp;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                float f = 0.f;
                if (v < nvec && k0 + c < r) {
                    f = (float)acc[c];
                    S_out[(i0 + i) * r + k0 + c] = f;
                }
                Ys[i * ld + k0 + c] = (double)f;
            }
        };
        // two vectors per thread and pass, so that at rp = 16 a thread has all its loads in flight at once (the kernel
        // is bound by the latency of these loads: the partials were written by the other XCDs)
        for (int v0 = tid; v0 < total_vec; v0 += 512) {
            const int v1 = v0 + 256;
            double acc0[4] = {0.0, 0.0, 0.0, 0.0}, acc1[4] = {0.0, 0.0, 0.0, 0.0};
            for (int sp0 = 0; sp0 < nsplit; sp0 += 16) {
                float4 x0[16], x1[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    const float4* src = reinterpret_cast<const float4*>(base + (int64_t)(sp0 + u) * d * rp);
                    x0[u] = (v0 < nvec && sp0 + u < nsplit) ? src[v0] : make_float4(0.f, 0.f, 0.f, 0.f);
                    x1[u] = (v1 < nvec && sp0 + u < nsplit) ? src[v1] : make_float4(0.f, 0.f, 0.f, 0.f);
                }
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    acc0[0] += (double)x0[u].x; acc0[1] += (double)x0[u].y;
                    acc0[2] += (double)x0[u].z; acc0[3] += (double)x0[u].w;
                    acc1[0] += (double)x1[u].x; acc1[1] += (double)x1[u].y;
                    acc1[2] += (double)x1[u].z; acc1[3] += (double)x1[u].w;
                }
            }
            finish(v0, acc0);
            if (v1 < total_vec) finish(v1, acc1);
        }
    } else {
        for (int e = tid; e < rows_pad * rp; e += 256) {
            const int i = e / rp, k = e % rp;
            const float v = (i < rows && k < r) ? S[(i0 + i) * r + k] : 0.f;
            Ys[i * ld + k] = (double)v;
        }
    }
    __syncthreads();
    gram_partial(Ys, ld, rows_pad, rp, partial, bx);
}

__global__ __launch_bounds__(256) void qr_gram_kernel(const float* __restrict__ S, const float* __restrict__ splits,
                                                      int nsplit, float* __restrict__ S_out, int64_t d, int r, int rp,
                                                      double* __restrict__ partial) {
    qr_gram_body(S, splits, nsplit, S_out, d, r, rp, partial, blockIdx.x);
}

// several factorisations per launch: per problem, what the three launches of one factorisation need
struct QrDev {
    const float* S; const float* splits; int nsplit; float* S_out; const float* Sin;
    int64_t d; int r; int nblk;
    double *Q1, *partial1, *partial2;
    float* Q; bf16_t* planes;
};
__global__ __launch_bounds__(256) void qr_gram_many_kernel(const KBatch<QrDev> tb, int rp) {
    uint32_t bx, by;
    const QrDev& a = tb.a[kbatch_find(tb, bx, by)];
    qr_gram_body(a.S, a.splits, a.nsplit, a.S_out, a.d, a.r, rp, a.partial1, bx);
}

// launch 2: R1 from the partials, Q1 = S R1^-1 for the block's rows (fp64, stored), Gram partials of Q1.
template <int RP>
__device__ __forceinline__ void qr_apply_gram_body(const float* __restrict__ S, int64_t d, int r,
                                                   const double* __restrict__ partial1, int nblk,
                                                   double* __restrict__ Q1, double* __restrict__ partial2, int* flag,
                                                   uint32_t bx) {
    extern __shared__ __align__(16) double qr_smem[];
    constexpr int rp = RP;
    const int ld = rp + 1;
    double* Ys = qr_smem;
    double* Gs = qr_smem + QR_ROWS * ld;
    const int tid = threadIdx.x;
    const int64_t i0 = (int64_t)bx * QR_ROWS;
    const int rows = (int)min((int64_t)QR_ROWS, d - i0);
    const int rows_pad = (rows + 3) & ~3;
    float y[RP];
    load_row_t<RP>(S + (i0 + min(tid, rows - 1)) * r, r, tid < rows, y);
    for (int e = tid; e < rows_pad * ld; e += 256) Ys[e] = 0.0;
    reduce_and_factor(partial1, nblk, Gs, r, rp, flag, bx);
    if (tid < rows) {
        double* q = Ys + tid * ld;
        solve_row_t<RP>(y, Gs, q);
        for (int c = 0; c < r; ++c) Q1[(i0 + tid) * r + c] = q[c];
    }
    __syncthreads();
    gram_partial(Ys, ld, rows_pad, rp, partial2, bx);
}

template <int RP>
__global__ __launch_bounds__(256) void qr_apply_gram_kernel(const float* __restrict__ S, int64_t d, int r,
                                                            const double* __restrict__ partial1, int nblk,
                                                            double* __restrict__ Q1, double* __restrict__ partial2,
                                                            int* flag) {
    qr_apply_gram_body<RP>(S, d, r, partial1, nblk, Q1, partial2, flag, blockIdx.x);
}

template <int RP>
__global__ __launch_bounds__(256) void qr_apply_gram_many_kernel(const KBatch<QrDev> tb, int* flag) {
    uint32_t bx, by;
    const QrDev& a = tb.a[kbatch_find(tb, bx, by)];
    qr_apply_gram_body<RP>(a.Sin, a.d, a.r, a.partial1, a.nblk, a.Q1, a.partial2, flag, bx);
}

// launch 3: Q = Q1 R2^-1, rounded to fp32; planes (nullable) receive the hi/mid/lo bf16 parts [3][rp][d].
// With Tin = float the same kernel closes a single-pass factorisation: Q = Y R1^-1 straight from launch 1's partials.
template <int RP, typename Tin>
__device__ __forceinline__ void qr_apply_final_body(const Tin* __restrict__ Q1, int64_t d, int r,
                                                    const double* __restrict__ partial2, int nblk,
                                                    float* __restrict__ Q, bf16_t* __restrict__ planes, int* flag,
                                                    uint32_t bx) {
    extern __shared__ __align__(16) double qr_smem[];
    constexpr int rp = RP;
    const int ld = rp + 1;
    double* Gs = qr_smem;                 // [rp][rp]
    double* Qs = qr_smem + rp * rp;       // [QR_ROWS][ld]
    const int tid = threadIdx.x;
    const int64_t i0 = (int64_t)bx * QR_ROWS;
    const int rows = (int)min((int64_t)QR_ROWS, d - i0);
    Tin y[RP];
    load_row_t<RP>(Q1 + (i0 + min(tid, rows - 1)) * r, r, tid < rows, y);
    reduce_and_factor(partial2, nblk, Gs, r, rp, flag, bx);
    if (tid < rows) {
        double* q = Qs + tid * ld;
        solve_row_t<RP>(y, Gs, q);
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

template <int RP, typename Tin>
__global__ __launch_bounds__(256) void qr_apply_final_kernel(const Tin* __restrict__ Q1, int64_t d, int r,
                                                             const double* __restrict__ partial2, int nblk,
                                                             float* __restrict__ Q, bf16_t* __restrict__ planes,
                                                             int* flag) {
    qr_apply_final_body<RP, Tin>(Q1, d, r, partial2, nblk, Q, planes, flag, blockIdx.x);
}

// DOUBLE_IN: second pass of CholeskyQR2 (input Q1, partials of Q1); otherwise the single-pass form (input Y)
template <int RP, bool DOUBLE_IN>
__global__ __launch_bounds__(256) void qr_apply_final_many_kernel(const KBatch<QrDev> tb, int* flag) {
    uint32_t bx, by;
    const QrDev& a = tb.a[kbatch_find(tb, bx, by)];
    if constexpr (DOUBLE_IN) qr_apply_final_body<RP, double>(a.Q1, a.d, a.r, a.partial2, a.nblk, a.Q, a.planes, flag, bx);
    else qr_apply_final_body<RP, float>(a.Sin, a.d, a.r, a.partial1, a.nblk, a.Q, a.planes, flag, bx);
}

// ---- r = 1 (the paper's operating point): the thin QR of a single column with a positive diagonal is the column
// divided by its norm, so the orthonormalisation is a sum of squares and a scaling: two small launches, no Gram
// matrix, no factorisation, and nothing for a second pass to refine.
constexpr int QR1_ROWS = 1024;   // rows per workgroup (4 per thread)

// launch 1: y_i = the column (or the fp64 sum of its partial sketches in split order, rounded to fp32 and stored to
// S_out like the general path does), partial[b] = sum of y_i^2 over the block's rows (fp64, fixed order)
__device__ __forceinline__ void qr1_sumsq_body(const float* __restrict__ S, const float* __restrict__ splits, int nsplit, int rp,
                                               float* __restrict__ S_out, int64_t d, double* __restrict__ partial, uint32_t bx) {
    __shared__ double red[4];
    const int tid = threadIdx.x;
    double ss = 0.0;
#pragma unroll
    for (int u = 0; u < QR1_ROWS / 256; ++u) {
        const int64_t i = (int64_t)bx * QR1_ROWS + u * 256 + tid;
        if (i >= d) continue;
        float y;
        if (splits != nullptr) {
            double acc = 0.0;
            for (int sp = 0; sp < nsplit; ++sp) acc += (double)splits[((int64_t)sp * d + i) * rp];
            y = (float)acc;
            S_out[i] = y;
        } else {
            y = S[i];
        }
        ss = fma((double)y, (double)y, ss);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    if (tid == 0) partial[bx] = (red[0] + red[1]) + (red[2] + red[3]);
}

// launch 2: q = y / sqrt(sum of the partials) -> Q fp32 [d][1] and, if asked, the bf16 planes [3][rp][d] (rows of the
// padding columns zero).  A sum that is not positive (an all-zero sketch) raises the numeric flag.
__device__ __forceinline__ void qr1_scale_body(const float* __restrict__ Y, int64_t d, int rp, const double* __restrict__ partial,
                                               int nblk, float* __restrict__ Q, bf16_t* __restrict__ planes, int* flag,
                                               uint32_t bx) {
    const int tid = threadIdx.x;
    double sum = 0.0;
    for (int b = 0; b < nblk; ++b) sum += partial[b];          // uniform: every thread adds the same few values
    if (!(sum > 0.0)) {
        if (tid == 0 && bx == 0) *flag = 1;
        sum = 1.0;
    }
    const double inv = 1.0 / sqrt(sum);
#pragma unroll
    for (int u = 0; u < QR1_ROWS / 256; ++u) {
        const int64_t i = (int64_t)bx * QR1_ROWS + u * 256 + tid;
        if (i >= d) continue;
        const float q = (float)((double)Y[i] * inv);
        Q[i] = q;
        if (planes != nullptr) {
            bf16_t hi, mid, lo;
            split3_bf16(q, hi, mid, lo);
            planes[((int64_t)0 * rp) * d + i] = hi;
            planes[((int64_t)1 * rp) * d + i] = mid;
            planes[((int64_t)2 * rp) * d + i] = lo;
            for (int c = 1; c < rp; ++c) {
                planes[((int64_t)0 * rp + c) * d + i] = 0;
                planes[((int64_t)1 * rp + c) * d + i] = 0;
                planes[((int64_t)2 * rp + c) * d + i] = 0;
            }
        }
    }
}

__global__ __launch_bounds__(256) void qr1_sumsq_kernel(const float* __restrict__ S, const float* __restrict__ splits, int nsplit,
                                                        int rp, float* __restrict__ S_out, int64_t d, double* __restrict__ partial) {
    qr1_sumsq_body(S, splits, nsplit, rp, S_out, d, partial, blockIdx.x);
}
__global__ __launch_bounds__(256) void qr1_scale_kernel(const float* __restrict__ Y, int64_t d, int rp,
                                                        const double* __restrict__ partial, int nblk, float* __restrict__ Q,
                                                        bf16_t* __restrict__ planes, int* flag) {
    qr1_scale_body(Y, d, rp, partial, nblk, Q, planes, flag, blockIdx.x);
}
__global__ __launch_bounds__(256) void qr1_sumsq_many_kernel(const KBatch<QrDev> tb, int rp) {
    uint32_t bx, by;
    const QrDev& a = tb.a[kbatch_find(tb, bx, by)];
    qr1_sumsq_body(a.S, a.splits, a.nsplit, rp, a.S_out, a.d, a.partial1, bx);
}
__global__ __launch_bounds__(256) void qr1_scale_many_kernel(const KBatch<QrDev> tb, int rp, int* flag) {
    uint32_t bx, by;
    const QrDev& a = tb.a[kbatch_find(tb, bx, by)];
    qr1_scale_body(a.Sin, a.d, rp, a.partial1, a.nblk, a.Q, a.planes, flag, bx);
}
static inline int64_t qr1_blocks(int64_t d) { return (d + QR1_ROWS - 1) / QR1_ROWS; }

// the launches after the first, for one padded rank (the rows' registers are sized by it)
template <int RP>
static hipError_t launch_apply(dim3 grid, size_t smem, hipStream_t st, const float* Sin, int64_t d, int r, const double* partial1,
                               double* partial2, int nblk, double* Q1, float* Q, bf16_t* planes, int* numeric_flag, bool refine) {
    static bool attr_set = false;
    if (!attr_set) {
        const int big = (QR_ROWS * (kMaxRank + 1) + kMaxRank * kMaxRank) * (int)sizeof(double);
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(qr_apply_gram_kernel<RP>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, big);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(qr_apply_final_kernel<RP, double>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, big);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(qr_apply_final_kernel<RP, float>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, big);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const dim3 block(256);
    if (!refine) {
        hipLaunchKernelGGL((qr_apply_final_kernel<RP, float>), grid, block, smem, st, Sin, d, r, partial1, nblk, Q, planes, numeric_flag);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(qr_apply_gram_kernel<RP>, grid, block, smem, st, Sin, d, r, partial1, nblk, Q1, partial2, numeric_flag);
    {
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((qr_apply_final_kernel<RP, double>), grid, block, smem, st, Q1, d, r, partial2, nblk, Q, planes, numeric_flag);
    return hipGetLastError();
}

hipError_t launch_qr(const float* S, const float* splits, int nsplit, int rp, float* S_out, int64_t d, int r, float* Q,
                     bf16_t* planes, void* workspace, int* numeric_flag, bool refine, hipStream_t st) {
    if (d == 0) return hipSuccess;
    if (r == 1) {
        const int nb1 = (int)qr1_blocks(d);
        double* part = reinterpret_cast<double*>(workspace);          // nb1 <= the d doubles reserved for Q1
        const float* Y = splits ? S_out : S;
        hipLaunchKernelGGL(qr1_sumsq_kernel, dim3((unsigned)nb1), dim3(256), 0, st, S, splits, nsplit, rp, S_out, d, part);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(qr1_scale_kernel, dim3((unsigned)nb1), dim3(256), 0, st, Y, d, rp, part, nb1, Q, planes, numeric_flag);
        return hipGetLastError();
    }
    const int nblk = (int)qr_blocks(d);
    double* Q1 = reinterpret_cast<double*>(workspace);
    double* partial1 = Q1 + d * r;
    double* partial2 = partial1 + (size_t)nblk * rp * rp;
    dim3 grid((unsigned)nblk), block(256);
    const size_t sm_full = ((size_t)QR_ROWS * (rp + 1) + (size_t)rp * rp) * sizeof(double);
    const float* Sin = splits ? S_out : S;
    static bool attr_set = false;
    if (!attr_set) {
        const int big = (QR_ROWS * (kMaxRank + 1) + kMaxRank * kMaxRank) * (int)sizeof(double);
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(qr_gram_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, big);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(qr_gram_kernel, grid, block, sm_full, st, S, splits, nsplit, S_out, d, r, rp, partial1);
    {
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;      // the launches below consume what this one would have written
    }
    switch (rp) {
        case 16: return launch_apply<16>(grid, sm_full, st, Sin, d, r, partial1, partial2, nblk, Q1, Q, planes, numeric_flag, refine);
        case 32: return launch_apply<32>(grid, sm_full, st, Sin, d, r, partial1, partial2, nblk, Q1, Q, planes, numeric_flag, refine);
        case 48: return launch_apply<48>(grid, sm_full, st, Sin, d, r, partial1, partial2, nblk, Q1, Q, planes, numeric_flag, refine);
        case 64: return launch_apply<64>(grid, sm_full, st, Sin, d, r, partial1, partial2, nblk, Q1, Q, planes, numeric_flag, refine);
        default: return hipErrorInvalidValue;
    }
}

template <int RP>
static hipError_t launch_apply_many(const KBatch<QrDev>& tb, unsigned blocks, size_t smem, int* flag, bool refine, hipStream_t st) {
    static bool attr_set = false;
    if (!attr_set) {
        const int big = (QR_ROWS * (kMaxRank + 1) + kMaxRank * kMaxRank) * (int)sizeof(double);
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(qr_apply_gram_many_kernel<RP>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, big);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(qr_apply_final_many_kernel<RP, true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, big);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(qr_apply_final_many_kernel<RP, false>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, big);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const dim3 grid(blocks), block(256);
    if (!refine) {
        hipLaunchKernelGGL((qr_apply_final_many_kernel<RP, false>), grid, block, smem, st, tb, flag);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(qr_apply_gram_many_kernel<RP>, grid, block, smem, st, tb, flag);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((qr_apply_final_many_kernel<RP, true>), grid, block, smem, st, tb, flag);
    return hipGetLastError();
}

hipError_t launch_qr_many(const QrArgs* a, int n, int* numeric_flag, bool refine, hipStream_t st) {
    if (n < 0 || n > kBatchMax) return hipErrorInvalidValue;
    KBatch<QrDev> tb;
    tb.n = 0;
    uint64_t blocks = 0;
    int rp = 0, rank1 = -1;
    for (int m = 0; m < n; ++m) {
        if (a[m].d == 0) continue;
        if (rp == 0) rp = a[m].rp;
        if (rank1 < 0) rank1 = (a[m].r == 1);
        // one padded rank per launch, and single columns (normalised, not factored) apart from the others
        if (a[m].rp != rp || (a[m].r == 1) != (rank1 == 1)) return hipErrorInvalidValue;
        QrDev q;
        q.S = a[m].S; q.splits = a[m].splits; q.nsplit = a[m].nsplit; q.S_out = a[m].S_out;
        q.Sin = a[m].splits ? a[m].S_out : a[m].S;
        q.d = a[m].d; q.r = a[m].r; q.nblk = (int)qr_blocks(a[m].d);
        q.Q1 = reinterpret_cast<double*>(a[m].workspace);
        q.partial1 = q.Q1 + a[m].d * a[m].r;
        q.partial2 = q.partial1 + (size_t)q.nblk * rp * rp;
        q.Q = a[m].Q; q.planes = a[m].planes;
        if (rank1 == 1) { q.nblk = (int)qr1_blocks(a[m].d); q.partial1 = q.Q1; }
        tb.first[tb.n] = (uint32_t)blocks; tb.gx[tb.n] = (uint32_t)q.nblk; tb.a[tb.n++] = q;
        blocks += (uint64_t)q.nblk;
    }
    if (tb.n == 0) return hipSuccess;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    if (rank1 == 1) {
        hipLaunchKernelGGL(qr1_sumsq_many_kernel, dim3((unsigned)blocks), dim3(256), 0, st, tb, rp);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(qr1_scale_many_kernel, dim3((unsigned)blocks), dim3(256), 0, st, tb, rp, numeric_flag);
        return hipGetLastError();
    }
    const size_t sm_full = ((size_t)QR_ROWS * (rp + 1) + (size_t)rp * rp) * sizeof(double);
    static bool attr_set = false;
    if (!attr_set) {
        const int big = (QR_ROWS * (kMaxRank + 1) + kMaxRank * kMaxRank) * (int)sizeof(double);
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(qr_gram_many_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, big);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(qr_gram_many_kernel, dim3((unsigned)blocks), dim3(256), sm_full, st, tb, rp);
    {
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    switch (rp) {
        case 16: return launch_apply_many<16>(tb, (unsigned)blocks, sm_full, numeric_flag, refine, st);
        case 32: return launch_apply_many<32>(tb, (unsigned)blocks, sm_full, numeric_flag, refine, st);
        case 48: return launch_apply_many<48>(tb, (unsigned)blocks, sm_full, numeric_flag, refine, st);
        case 64: return launch_apply_many<64>(tb, (unsigned)blocks, sm_full, numeric_flag, refine, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace agzo
