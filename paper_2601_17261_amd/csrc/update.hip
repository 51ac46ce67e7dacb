// In-place rank-r sweep of Alg. 2 (restore / update line, Eq. 10):
//     W[i][j] -= lr * g * sum_k G[i][k] * B[j][k]
// W is read and written exactly once (HBM-bound); G is regenerated from the Philox seed per tile
// and never stored; B (d_in x r fp32) is small and stays in L2.  fp32 arithmetic, one rounding
// to the storage type on the store.
#include "agzo_internal.h"

namespace agzo {

constexpr int UP_TI = 64;    // rows (d_out) per tile
constexpr int UP_TJ = 256;   // cols (d_in) per tile
constexpr int UP_TR = 8;     // rows per thread

// KC = number of k handled per register chunk; nchunk chunks cover r (zero padded)
template <int KC, bool BF16>
__global__ __launch_bounds__(256) void update_kernel(void* __restrict__ Wv, int64_t ldw, int64_t d_out, int64_t d_in,
                                                     const float* __restrict__ B, int r, int nchunk, uint32_t s_lo,
                                                     uint32_t s_hi, float lr, const double* __restrict__ g_dev) {
    extern __shared__ __align__(16) float up_smem[];
    const int rp = KC * nchunk;
    float* Gs = up_smem;                 // [UP_TI][rp]
    float* Bt = up_smem + UP_TI * rp;    // [rp][UP_TJ]  (transposed: k-major)
    const int tid = threadIdx.x;
    const int64_t i0 = (int64_t)blockIdx.y * UP_TI, j0 = (int64_t)blockIdx.x * UP_TJ;

    // G tile from the seed: one Philox call = 4 columns of one row
    const int nquad = (rp + 3) / 4;
    for (int e = tid; e < UP_TI * nquad; e += 256) {
        const int ii = e / nquad, q = e % nquad;
        float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
        if (i0 + ii < d_out && q * 4 < r) z = philox_normal4(s_lo, s_hi, AGZO_TAG_G, (uint32_t)(i0 + ii), (uint32_t)q);
        const float v[4] = {z.x, z.y, z.z, z.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int k = q * 4 + c;
            if (k < rp) Gs[ii * rp + k] = (k < r) ? v[c] : 0.f;
        }
    }
    for (int e = tid; e < UP_TJ * rp; e += 256) {
        const int jj = e / rp, k = e % rp;
        Bt[k * UP_TJ + jj] = (j0 + jj < d_in && k < r) ? B[(j0 + jj) * r + k] : 0.f;
    }
    __syncthreads();

    const float coef = -lr * (g_dev ? (float)(*g_dev) : 1.0f);
    const int tx = tid & 31;          // 8 consecutive columns
    const int ty = tid >> 5;          // rows ty + 8*s
    const int64_t jc = j0 + tx * 8;

    float acc[UP_TR][8];
#pragma unroll
    for (int s = 0; s < UP_TR; ++s)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[s][c] = 0.f;

    for (int ch = 0; ch < nchunk; ++ch) {
        float b[KC][8];
#pragma unroll
        for (int k = 0; k < KC; ++k) {
            const float4 lo = *reinterpret_cast<const float4*>(&Bt[(ch * KC + k) * UP_TJ + tx * 8]);
            const float4 hi = *reinterpret_cast<const float4*>(&Bt[(ch * KC + k) * UP_TJ + tx * 8 + 4]);
            b[k][0] = lo.x; b[k][1] = lo.y; b[k][2] = lo.z; b[k][3] = lo.w;
            b[k][4] = hi.x; b[k][5] = hi.y; b[k][6] = hi.z; b[k][7] = hi.w;
        }
#pragma unroll
        for (int s = 0; s < UP_TR; ++s) {
            const float* g = &Gs[(ty + 8 * s) * rp + ch * KC];
#pragma unroll
            for (int k = 0; k < KC; ++k) {
                const float gv = g[k];
#pragma unroll
                for (int c = 0; c < 8; ++c) acc[s][c] = fmaf(gv, b[k][c], acc[s][c]);
            }
        }
    }

    if (jc >= d_in) return;
    const bool full = (jc + 8 <= d_in);
#pragma unroll
    for (int s = 0; s < UP_TR; ++s) {
        const int64_t i = i0 + ty + 8 * s;
        if (i >= d_out) continue;
        if (BF16) {
            bf16_t* w = reinterpret_cast<bf16_t*>(Wv) + i * ldw + jc;
            if (full) {
                uint4 raw = *reinterpret_cast<const uint4*>(w);
                uint32_t* pw = reinterpret_cast<uint32_t*>(&raw);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float w0 = __uint_as_float(pw[q] << 16), w1 = __uint_as_float(pw[q] & 0xFFFF0000u);
                    const bf16_t o0 = f32_to_bf16(fmaf(coef, acc[s][2 * q], w0));
                    const bf16_t o1 = f32_to_bf16(fmaf(coef, acc[s][2 * q + 1], w1));
                    pw[q] = (uint32_t)o0 | ((uint32_t)o1 << 16);
                }
                *reinterpret_cast<uint4*>(w) = raw;
            } else {
                for (int c = 0; c < 8 && jc + c < d_in; ++c) w[c] = f32_to_bf16(fmaf(coef, acc[s][c], bf16_to_f32(w[c])));
            }
        } else {
            float* w = reinterpret_cast<float*>(Wv) + i * ldw + jc;
            if (full && ((reinterpret_cast<uintptr_t>(w) & 15) == 0)) {
                float4 a = *reinterpret_cast<const float4*>(w), c4 = *reinterpret_cast<const float4*>(w + 4);
                a.x = fmaf(coef, acc[s][0], a.x); a.y = fmaf(coef, acc[s][1], a.y);
                a.z = fmaf(coef, acc[s][2], a.z); a.w = fmaf(coef, acc[s][3], a.w);
                c4.x = fmaf(coef, acc[s][4], c4.x); c4.y = fmaf(coef, acc[s][5], c4.y);
                c4.z = fmaf(coef, acc[s][6], c4.z); c4.w = fmaf(coef, acc[s][7], c4.w);
                *reinterpret_cast<float4*>(w) = a;
                *reinterpret_cast<float4*>(w + 4) = c4;
            } else {
                for (int c = 0; c < 8 && jc + c < d_in; ++c) w[c] = fmaf(coef, acc[s][c], w[c]);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// r > 8: the outer product G B^T runs on the matrix cores (v_mfma_f32_32x32x16_bf16, K = r padded to 16).
// Roles: A-operand rows = basis rows (columns j of W, permuted so that a lane ends up with 16 consecutive
// j), B-operand rows = G rows (rows i of W).  G and B are split hi + lo in bf16 and the products hi*hi,
// hi*lo, lo*hi are accumulated: relative error 2^-16 of the increment.  A wave owns 32 rows x 256 columns.
// ---------------------------------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
union FragU {
    uint4 u;
    bf16x8 v;
};

__device__ __forceinline__ int upd_perm(int m) { return ((m >> 2) & 1) * 16 + ((m >> 3) & 3) * 4 + (m & 3); }

// eight fp32 values -> hi and lo bf16 fragments
__device__ __forceinline__ void split_frag(const float (&f)[8], FragU& hi, FragU& lo) {
    uint32_t h[4] = {0, 0, 0, 0}, l[4] = {0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const bf16_t a = f32_to_bf16(f[i]);
        const bf16_t b = f32_to_bf16(f[i] - bf16_to_f32(a));
        h[i >> 1] |= ((uint32_t)a) << ((i & 1) * 16);
        l[i >> 1] |= ((uint32_t)b) << ((i & 1) * 16);
    }
    hi.u = make_uint4(h[0], h[1], h[2], h[3]);
    lo.u = make_uint4(l[0], l[1], l[2], l[3]);
}

constexpr int UM_ROWS = 32;            // rows of W per workgroup
constexpr int UM_COLS_PER_WAVE = 256;  // columns per wave (8 blocks of 32)

template <int NK, bool BF16>   // NK = rp / 16
__global__ __launch_bounds__(256) void update_mfma_kernel(void* __restrict__ Wv, int64_t ldw, int64_t d_out, int64_t d_in,
                                                          const float* __restrict__ B, int r, uint32_t s_lo,
                                                          uint32_t s_hi, float lr, const double* __restrict__ g_dev) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lr_ = lane & 31, lh = lane >> 5;
    const int64_t i0 = (int64_t)blockIdx.y * UM_ROWS;
    const int64_t jw = ((int64_t)blockIdx.x * 4 + wave) * UM_COLS_PER_WAVE;
    if (jw >= d_in) return;
    const float coef = -lr * (g_dev ? (float)(*g_dev) : 1.0f);
    const int64_t i = i0 + lr_;

    // G fragments of this lane's row: k = 16*kc + 8*lh .. +7
    FragU gh[NK], gl[NK];
#pragma unroll
    for (int kc = 0; kc < NK; ++kc) {
        const int k0 = 16 * kc + 8 * lh;
        float g[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (i < d_out) {
            if (k0 < r) {
                const float4 z = philox_normal4(s_lo, s_hi, AGZO_TAG_G, (uint32_t)i, (uint32_t)(k0 >> 2));
                g[0] = z.x; g[1] = z.y; g[2] = z.z; g[3] = z.w;
            }
            if (k0 + 4 < r) {
                const float4 z = philox_normal4(s_lo, s_hi, AGZO_TAG_G, (uint32_t)i, (uint32_t)((k0 >> 2) + 1));
                g[4] = z.x; g[5] = z.y; g[6] = z.z; g[7] = z.w;
            }
#pragma unroll
            for (int q = 0; q < 8; ++q)
                if (k0 + q >= r) g[q] = 0.f;
        }
        split_frag(g, gh[kc], gl[kc]);
    }

    for (int jb = 0; jb < UM_COLS_PER_WAVE / 32; ++jb) {
        const int64_t j0 = jw + jb * 32;
        if (j0 >= d_in) break;
        floatx16 z;
#pragma unroll
        for (int e = 0; e < 16; ++e) z[e] = 0.f;
        const int64_t jrow = j0 + upd_perm(lr_);     // basis row this lane feeds as A-operand row lr_
#pragma unroll
        for (int kc = 0; kc < NK; ++kc) {
            const int k0 = 16 * kc + 8 * lh;
            float b[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) b[q] = (jrow < d_in && k0 + q < r) ? B[jrow * r + k0 + q] : 0.f;
            FragU bh, bl;
            split_frag(b, bh, bl);
            z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bh.v, gh[kc].v, z, 0, 0, 0);
            z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bh.v, gl[kc].v, z, 0, 0, 0);
            z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bl.v, gh[kc].v, z, 0, 0, 0);
        }
        if (i >= d_out) continue;
        const int64_t jc = j0 + 16 * lh;             // this lane's 16 consecutive columns of row i
        if (BF16) {
            bf16_t* w = reinterpret_cast<bf16_t*>(Wv) + i * ldw + jc;
#pragma unroll
            for (int hq = 0; hq < 2; ++hq) {
                if (jc + 8 * hq >= d_in) continue;   // d_in is a multiple of 8: an 8-column piece is all in or all out
                uint4 raw = *reinterpret_cast<const uint4*>(w + 8 * hq);
                uint32_t* pw = reinterpret_cast<uint32_t*>(&raw);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float w0 = __uint_as_float(pw[q] << 16), w1 = __uint_as_float(pw[q] & 0xFFFF0000u);
                    const bf16_t o0 = f32_to_bf16(fmaf(coef, z[8 * hq + 2 * q], w0));
                    const bf16_t o1 = f32_to_bf16(fmaf(coef, z[8 * hq + 2 * q + 1], w1));
                    pw[q] = (uint32_t)o0 | ((uint32_t)o1 << 16);
                }
                *reinterpret_cast<uint4*>(w + 8 * hq) = raw;
            }
        } else {
            float* w = reinterpret_cast<float*>(Wv) + i * ldw + jc;
#pragma unroll
            for (int e = 0; e < 16; ++e)
                if (jc + e < d_in) w[e] = fmaf(coef, z[e], w[e]);
        }
    }
}

template <int NK>
static hipError_t launch_mfma(void* W, int dtype, int64_t ldw, int64_t d_out, int64_t d_in, const float* B, int r,
                              uint64_t seed, float lr, const double* g_dev, hipStream_t st) {
    dim3 grid((unsigned)((d_in + 4 * UM_COLS_PER_WAVE - 1) / (4 * UM_COLS_PER_WAVE)), (unsigned)((d_out + UM_ROWS - 1) / UM_ROWS));
    if (dtype == AGZO_BF16)
        hipLaunchKernelGGL((update_mfma_kernel<NK, true>), grid, dim3(256), 0, st, W, ldw, d_out, d_in, B, r, (uint32_t)seed,
                           (uint32_t)(seed >> 32), lr, g_dev);
    else
        hipLaunchKernelGGL((update_mfma_kernel<NK, false>), grid, dim3(256), 0, st, W, ldw, d_out, d_in, B, r,
                           (uint32_t)seed, (uint32_t)(seed >> 32), lr, g_dev);
    return hipGetLastError();
}

template <int KC>
static hipError_t launch_kc(void* W, int dtype, int64_t ldw, int64_t d_out, int64_t d_in, const float* B, int r,
                            int nchunk, uint64_t seed, float lr, const double* g_dev, hipStream_t st) {
    dim3 grid((unsigned)((d_in + UP_TJ - 1) / UP_TJ), (unsigned)((d_out + UP_TI - 1) / UP_TI));
    const int rp = KC * nchunk;
    const size_t smem = (size_t)(UP_TI + UP_TJ) * rp * sizeof(float);
    if (dtype == AGZO_BF16) {
        static bool set = false;
        if (!set) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(update_kernel<KC, true>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize,
                                               (UP_TI + UP_TJ) * kMaxRank * (int)sizeof(float));
            if (e != hipSuccess) return e;
            set = true;
        }
        hipLaunchKernelGGL((update_kernel<KC, true>), grid, dim3(256), smem, st, W, ldw, d_out, d_in, B, r, nchunk,
                           (uint32_t)seed, (uint32_t)(seed >> 32), lr, g_dev);
    } else {
        static bool set = false;
        if (!set) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(update_kernel<KC, false>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize,
                                               (UP_TI + UP_TJ) * kMaxRank * (int)sizeof(float));
            if (e != hipSuccess) return e;
            set = true;
        }
        hipLaunchKernelGGL((update_kernel<KC, false>), grid, dim3(256), smem, st, W, ldw, d_out, d_in, B, r, nchunk,
                           (uint32_t)seed, (uint32_t)(seed >> 32), lr, g_dev);
    }
    return hipGetLastError();
}

hipError_t launch_update(void* W, int dtype, int64_t ldw, int64_t d_out, int64_t d_in, const float* B, int r,
                         uint64_t seed, float lr, const double* g_dev, hipStream_t st) {
    if (d_out == 0 || d_in == 0) return hipSuccess;
    if (r <= 1) return launch_kc<1>(W, dtype, ldw, d_out, d_in, B, r, 1, seed, lr, g_dev, st);
    if (r <= 2) return launch_kc<2>(W, dtype, ldw, d_out, d_in, B, r, 1, seed, lr, g_dev, st);
    if (r <= 4) return launch_kc<4>(W, dtype, ldw, d_out, d_in, B, r, 1, seed, lr, g_dev, st);
    if (r <= 8) return launch_kc<8>(W, dtype, ldw, d_out, d_in, B, r, 1, seed, lr, g_dev, st);
    // fp32 storage keeps exact fp32 products (VALU); bf16 storage takes the matrix-core outer product
    if (dtype != AGZO_BF16) return launch_kc<16>(W, dtype, ldw, d_out, d_in, B, r, (r + 15) / 16, seed, lr, g_dev, st);
    switch ((r + 15) / 16) {
        case 1: return launch_mfma<1>(W, dtype, ldw, d_out, d_in, B, r, seed, lr, g_dev, st);
        case 2: return launch_mfma<2>(W, dtype, ldw, d_out, d_in, B, r, seed, lr, g_dev, st);
        case 3: return launch_mfma<3>(W, dtype, ldw, d_out, d_in, B, r, seed, lr, g_dev, st);
        default: return launch_mfma<4>(W, dtype, ldw, d_out, d_in, B, r, seed, lr, g_dev, st);
    }
}

}  // namespace agzo
