// fp32-storage path: a generic strided GEMM whose products are accumulated in fp64 on the vector
// ALUs (CDNA4 issues fp64 FMA at the plain-fp32 rate), and the epilogue that adds the rank-r
// perturbation term eps * (X B) G^T (Eq. 7, factored) and reduces the loss.  Used for every
// product of the fp32 configuration: Y = X W^T, T = X Q, S = X^T T, S = X^T Omega.
#include "agzo_internal.h"

namespace agzo {

constexpr int TS = 64;   // C tile is TS x TS
constexpr int TK = 16;

// C[m][n] = sum_k A[m*sam + k*sak] * B[k*sbk + n*sbn]
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A, int64_t sam, int64_t sak,
                                                       const float* __restrict__ B, int64_t sbk, int64_t sbn,
                                                       float* __restrict__ C, int64_t ldc, int64_t M, int64_t N,
                                                       int64_t K) {
    __shared__ float As[TK][TS + 4];
    __shared__ float Bs[TK][TS + 4];
    const int tid = threadIdx.x;
    const int64_t m0 = (int64_t)blockIdx.y * TS, n0 = (int64_t)blockIdx.x * TS;
    const int tx = tid % 16, ty = tid / 16;
    double acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;

    // loader mapping: choose the index that is contiguous in memory to run fastest over threads
    const bool a_k_fast = (sak == 1);
    const bool b_k_fast = (sbk == 1);
    for (int64_t k0 = 0; k0 < K; k0 += TK) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            int e = tid + q * 256;  // 0..1023
            int mm, kk;
            if (a_k_fast) { kk = e % TK; mm = e / TK; } else { mm = e % TS; kk = e / TS; }
            int64_t gm = m0 + mm, gk = k0 + kk;
            As[kk][mm] = (gm < M && gk < K) ? A[gm * sam + gk * sak] : 0.f;
            int nn;
            if (b_k_fast) { kk = e % TK; nn = e / TK; } else { nn = e % TS; kk = e / TS; }
            int64_t gn = n0 + nn;
            gk = k0 + kk;
            Bs[kk][nn] = (gn < N && gk < K) ? B[gk * sbk + gn * sbn] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < TK; ++kk) {
            double a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = (double)As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = (double)Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fma(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int64_t gm = m0 + ty * 4 + i;
        if (gm >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int64_t gn = n0 + tx * 4 + j;
            if (gn < N) C[gm * ldc + gn] = (float)acc[i][j];
        }
    }
}

hipError_t launch_gemm_f32(const float* A, int64_t sam, int64_t sak, const float* B, int64_t sbk, int64_t sbn,
                           float* C, int64_t ldc, int64_t M, int64_t N, int64_t K, hipStream_t st) {
    if (M == 0 || N == 0) return hipSuccess;
    dim3 grid((unsigned)((N + TS - 1) / TS), (unsigned)((M + TS - 1) / TS));
    hipLaunchKernelGGL(gemm_f32_kernel, grid, dim3(256), 0, st, A, sam, sak, B, sbk, sbn, C, ldc, M, N, K);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// epilogue: tile of EP_T tokens x EP_J outputs per workgroup
// ---------------------------------------------------------------------------
constexpr int EP_T = 32;
constexpr int EP_J = 64;

int epilogue_f32_num_workgroups(int64_t M, int64_t N) {
    return (int)(((M + EP_T - 1) / EP_T) * ((N + EP_J - 1) / EP_J));
}

__global__ __launch_bounds__(256) void epilogue_f32_kernel(float* __restrict__ Y, int64_t ldy, int64_t M, int64_t N,
                                                           const float* __restrict__ P, int r, float eps_signed,
                                                           uint32_t s_lo, uint32_t s_hi, int loss_kind,
                                                           int target_dtype, const void* __restrict__ target,
                                                           int64_t ldt, double* __restrict__ partials) {
    __shared__ float Gs[EP_J][kMaxRank + 1];
    __shared__ float Ps[EP_T][kMaxRank + 1];
    __shared__ double red[256];
    const int tid = threadIdx.x;
    const int64_t t0 = (int64_t)blockIdx.y * EP_T, j0 = (int64_t)blockIdx.x * EP_J;
    if (P != nullptr) {
        const int nquad = (r + 3) / 4;
        for (int e = tid; e < EP_J * nquad; e += 256) {
            int jj = e / nquad, q = e % nquad;
            int64_t j = j0 + jj;
            float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
            if (j < N) z = philox_normal4(s_lo, s_hi, AGZO_TAG_G, (uint32_t)j, (uint32_t)q);
            float v[4] = {z.x, z.y, z.z, z.w};
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (q * 4 + i < r) Gs[jj][q * 4 + i] = v[i];
        }
        for (int e = tid; e < EP_T * r; e += 256) {
            int tt = e / r, k = e % r;
            int64_t t = t0 + tt;
            Ps[tt][k] = (t < M) ? P[t * r + k] : 0.f;
        }
        __syncthreads();
    }
    double part = 0.0;
    const int jj = tid % EP_J;
    const int64_t j = j0 + jj;
    for (int tt = tid / EP_J; tt < EP_T; tt += 256 / EP_J) {
        int64_t t = t0 + tt;
        if (t >= M || j >= N) continue;
        double y = (double)Y[t * ldy + j];
        if (P != nullptr) {
            double d = 0.0;
            for (int k = 0; k < r; ++k) d = fma((double)Ps[tt][k], (double)Gs[jj][k], d);
            y += (double)eps_signed * d;
            Y[t * ldy + j] = (float)y;
        }
        if (loss_kind == AGZO_LOSS_MSE) {
            float tv = (target_dtype == AGZO_BF16)
                           ? bf16_to_f32(reinterpret_cast<const bf16_t*>(target)[t * ldt + j])
                           : reinterpret_cast<const float*>(target)[t * ldt + j];
            double d = y - (double)tv;
            part = fma(d, d, part);
        }
    }
    if (loss_kind == AGZO_LOSS_MSE) {
        red[tid] = part;
        __syncthreads();
        for (int s = 128; s > 0; s >>= 1) {
            if (tid < s) red[tid] += red[tid + s];
            __syncthreads();
        }
        if (tid == 0) partials[(int64_t)blockIdx.y * gridDim.x + blockIdx.x] = red[0];
    }
}

hipError_t launch_epilogue_f32(float* Y, int64_t ldy, int64_t M, int64_t N, const float* P, int r, float eps_signed,
                               uint64_t seed, const GemmLossArgs& loss, hipStream_t st) {
    if (M == 0 || N == 0) return hipSuccess;
    if (P == nullptr && loss.kind != AGZO_LOSS_MSE) return hipSuccess;
    dim3 grid((unsigned)((N + EP_J - 1) / EP_J), (unsigned)((M + EP_T - 1) / EP_T));
    hipLaunchKernelGGL(epilogue_f32_kernel, grid, dim3(256), 0, st, Y, ldy, M, N, P, r, eps_signed, (uint32_t)seed,
                       (uint32_t)(seed >> 32), loss.kind, loss.target_dtype, loss.target, loss.ldt, loss.partials);
    return hipGetLastError();
}

}  // namespace agzo
