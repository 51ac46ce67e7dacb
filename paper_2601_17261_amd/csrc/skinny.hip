// Tall-skinny products of Alg. 1 on bf16 activations (HBM-bound sweeps of X):
//   xq  : T = X Q          (N x r), contraction over d_in   -> also used for the projection P = X B
//   xtt : S = X^T T        (d_in x r), contraction over tokens (T = Omega or T = X Q)
// X is bf16; the small fp32 factor (Q, B, T, Omega) enters the matrix cores as three bf16 planes
// hi + mid + lo, whose sum is the fp32 value, so the products carry fp32-level accuracy while the
// kernels stay bound by the single read of X.  v_mfma_f32_16x16x32_bf16 throughout.
#include "agzo_internal.h"

namespace agzo {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

union Frag {
    uint4 u;
    bf16x8 v;
};

// ---------------------------------------------------------------------------
// xq: workgroup = 32 tokens, its 4 waves split d_in; partial tiles are summed through LDS.
// MFMA roles: A = X tile (rows = tokens, K = d_in), B = Q planes (K = d_in, cols = k).
// ---------------------------------------------------------------------------
constexpr int XQ_TOK = 32;

template <int NB>
__global__ __launch_bounds__(256) void xq_bf16_kernel(const bf16_t* __restrict__ X, int64_t ldx, int64_t M, int64_t K,
                                                      const bf16_t* __restrict__ Qpack, int r, float* __restrict__ T,
                                                      bf16_t* __restrict__ TpackT, int64_t m_pad) {
    constexpr int RP = NB * 16;
    __shared__ float red[4][XQ_TOK][RP + 1];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lm = lane & 15, lg = lane >> 4;
    const int64_t t0 = (int64_t)blockIdx.x * XQ_TOK;

    floatx4 acc[2][NB];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[mt][nb] = floatx4{0.f, 0.f, 0.f, 0.f};

    const int64_t ksteps = (K + 31) / 32;
    const int64_t per = (ksteps + 3) / 4;
    const int64_t s_begin = wave * per, s_end = min(s_begin + per, ksteps);
    const bf16_t* xrow[2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) xrow[mt] = X + min(t0 + mt * 16 + lm, M - 1) * ldx;

#pragma unroll 2
    for (int64_t s = s_begin; s < s_end; ++s) {
        const int64_t d = s * 32 + lg * 8;
        const bool in = d < K;
        Frag a[2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
            a[mt].u = in ? *reinterpret_cast<const uint4*>(xrow[mt] + d) : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
            for (int pl = 0; pl < 3; ++pl) {
                Frag b;
                b.u = in ? *reinterpret_cast<const uint4*>(Qpack + ((int64_t)(pl * RP + nb * 16 + lm)) * K + d)
                         : make_uint4(0, 0, 0, 0);
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
                    acc[mt][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[mt].v, b.v, acc[mt][nb], 0, 0, 0);
            }
        }
    }
    // D layout: row (token) = 4*(lane/16) + e, col (k) = lane%16
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int e = 0; e < 4; ++e) red[wave][mt * 16 + lg * 4 + e][nb * 16 + lm] = acc[mt][nb][e];
    __syncthreads();
    for (int idx = tid; idx < XQ_TOK * RP; idx += 256) {
        const int tt = idx % XQ_TOK, k = idx / XQ_TOK;
        const int64_t t = t0 + tt;
        const float v = (red[0][tt][k] + red[1][tt][k]) + (red[2][tt][k] + red[3][tt][k]);
        if (t < M && k < r && T != nullptr) T[t * r + k] = v;
        if (TpackT != nullptr && t < m_pad) {
            bf16_t hi, mid, lo;
            split3_bf16((t < M && k < r) ? v : 0.f, hi, mid, lo);
            TpackT[((int64_t)0 * RP + k) * m_pad + t] = hi;
            TpackT[((int64_t)1 * RP + k) * m_pad + t] = mid;
            TpackT[((int64_t)2 * RP + k) * m_pad + t] = lo;
        }
    }
}

hipError_t launch_xq_bf16(const bf16_t* X, int64_t ldx, int64_t M, int64_t K, const bf16_t* Qpack, int r, int rp,
                          float* T, bf16_t* TpackT, int64_t m_pad, hipStream_t st) {
    if (M == 0) return hipSuccess;
    // cover the padded token range too so that the planes' tail is zeroed
    const int64_t rows = TpackT ? m_pad : M;
    dim3 grid((unsigned)((rows + XQ_TOK - 1) / XQ_TOK));
    switch (rp / 16) {
        case 1: hipLaunchKernelGGL(xq_bf16_kernel<1>, grid, dim3(256), 0, st, X, ldx, M, K, Qpack, r, T, TpackT, m_pad); break;
        case 2: hipLaunchKernelGGL(xq_bf16_kernel<2>, grid, dim3(256), 0, st, X, ldx, M, K, Qpack, r, T, TpackT, m_pad); break;
        case 3: hipLaunchKernelGGL(xq_bf16_kernel<3>, grid, dim3(256), 0, st, X, ldx, M, K, Qpack, r, T, TpackT, m_pad); break;
        case 4: hipLaunchKernelGGL(xq_bf16_kernel<4>, grid, dim3(256), 0, st, X, ldx, M, K, Qpack, r, T, TpackT, m_pad); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// xtt: workgroup = (panel of 128 features) x (token range); waves interleave 32-token steps.
// MFMA roles: A = T^T planes (rows = k, K = tokens), B = X^T (K = tokens, cols = features).
// X is row-major in features, so a lane loads 8 features x 8 tokens as eight 16-byte rows and
// transposes them in registers (byte permutes) into eight token-contiguous operands.
// ---------------------------------------------------------------------------
constexpr int XTT_PANEL = 128;
constexpr int XTT_STEP = 32;

int xtt_num_splits(int64_t M, int64_t K) {
    const int64_t panels = (K + XTT_PANEL - 1) / XTT_PANEL;
    int64_t want = (256 + panels - 1) / panels;   // about one workgroup per CU; few splits keep the partials small
    const int64_t max_splits = (M + 4 * XTT_STEP - 1) / (4 * XTT_STEP);
    if (want > max_splits) want = max_splits;
    if (want < 1) want = 1;
    if (want > 16) want = 16;
    return (int)want;
}

template <int NB>
__global__ __launch_bounds__(256) void xtt_bf16_kernel(const bf16_t* __restrict__ X, int64_t ldx, int64_t M, int64_t K,
                                                       const bf16_t* __restrict__ TpackT, int64_t m_pad,
                                                       float* __restrict__ partial, int64_t tok_per_split) {
    constexpr int RP = NB * 16;
    extern __shared__ __align__(16) float sbuf[];   // [XTT_PANEL][RP]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lc = lane & 15, lg = lane >> 4;
    const int64_t db = (int64_t)blockIdx.x * XTT_PANEL;
    const int split = blockIdx.y;
    const int64_t ts = (int64_t)split * tok_per_split;
    const int64_t te = min(ts + tok_per_split, m_pad);

    floatx4 acc[NB][8];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[nb][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    const int64_t dcol = db + lc * 8;
    const bool din = dcol < K;
    for (int64_t tb = ts + wave * XTT_STEP; tb < te; tb += 4 * XTT_STEP) {
        uint4 v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int64_t t = min(tb + lg * 8 + i, M - 1);   // rows past M meet zero planes
            v[i] = din ? *reinterpret_cast<const uint4*>(X + t * ldx + dcol) : make_uint4(0, 0, 0, 0);
        }
        Frag a[NB][3];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int pl = 0; pl < 3; ++pl)
                a[nb][pl].u = *reinterpret_cast<const uint4*>(TpackT + ((int64_t)(pl * RP + nb * 16 + lc)) * m_pad + tb + lg * 8);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            // word q of v[i] holds features 2q (low half) and 2q+1 (high half) of token i
            const uint32_t sel = (j & 1) ? 0x07060302u : 0x05040100u;
            const int q = j >> 1;
            Frag b;
            const uint32_t* w0 = reinterpret_cast<const uint32_t*>(&v[0]);
            uint32_t o[4];
#pragma unroll
            for (int pp = 0; pp < 4; ++pp)
                o[pp] = __builtin_amdgcn_perm(w0[(2 * pp + 1) * 4 + q], w0[(2 * pp) * 4 + q], sel);
            b.u = make_uint4(o[0], o[1], o[2], o[3]);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int pl = 0; pl < 3; ++pl)
                    acc[nb][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[nb][pl].v, b.v, acc[nb][j], 0, 0, 0);
        }
    }
    // D layout: row (k within block) = 4*(lane/16) + e, col = lane%16 -> feature db + 8*lc + j
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int j = 0; j < 8; ++j)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float* dst = &sbuf[(lc * 8 + j) * RP + nb * 16 + lg * 4 + e];
                        if (w == 0) *dst = acc[nb][j][e]; else *dst += acc[nb][j][e];
                    }
        }
        __syncthreads();
    }
    float* out = partial + ((int64_t)split * K + db) * RP;
    const int64_t nvalid = min((int64_t)XTT_PANEL, K - db) * RP;
    for (int idx = tid; idx < XTT_PANEL * RP; idx += 256)
        if (idx < nvalid) out[idx] = sbuf[idx];
}

hipError_t launch_xtt_bf16(const bf16_t* X, int64_t ldx, int64_t M, int64_t K, const bf16_t* TpackT, int64_t m_pad,
                           int rp, float* partial, int nsplit, hipStream_t st) {
    if (M == 0 || K == 0) return hipSuccess;
    int64_t tok_per_split = (m_pad + nsplit - 1) / nsplit;
    tok_per_split = (tok_per_split + 4 * XTT_STEP - 1) / (4 * XTT_STEP) * (4 * XTT_STEP);
    dim3 grid((unsigned)((K + XTT_PANEL - 1) / XTT_PANEL), (unsigned)nsplit);
    const size_t smem = (size_t)XTT_PANEL * rp * sizeof(float);
    switch (rp / 16) {
        case 1: hipLaunchKernelGGL(xtt_bf16_kernel<1>, grid, dim3(256), smem, st, X, ldx, M, K, TpackT, m_pad, partial, tok_per_split); break;
        case 2: hipLaunchKernelGGL(xtt_bf16_kernel<2>, grid, dim3(256), smem, st, X, ldx, M, K, TpackT, m_pad, partial, tok_per_split); break;
        case 3: hipLaunchKernelGGL(xtt_bf16_kernel<3>, grid, dim3(256), smem, st, X, ldx, M, K, TpackT, m_pad, partial, tok_per_split); break;
        case 4: hipLaunchKernelGGL(xtt_bf16_kernel<4>, grid, dim3(256), smem, st, X, ldx, M, K, TpackT, m_pad, partial, tok_per_split); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// S[d][k] = sum over splits (fp64, fixed order) of partial[s][d][rp]
__global__ __launch_bounds__(256) void reduce_splits_kernel(const float* __restrict__ partial, int nsplit, int64_t d,
                                                            int rp, int r, float* __restrict__ S) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= d * rp) return;
    const int k = (int)(idx % rp);
    const int64_t row = idx / rp;
    if (k >= r) return;
    double s = 0.0;
    for (int sp = 0; sp < nsplit; ++sp) s += (double)partial[(int64_t)sp * d * rp + idx];
    S[row * r + k] = (float)s;
}

hipError_t launch_reduce_splits(const float* partial, int nsplit, int64_t d, int rp, int r, float* S, hipStream_t st) {
    if (d == 0) return hipSuccess;
    dim3 grid((unsigned)((d * rp + 255) / 256));
    hipLaunchKernelGGL(reduce_splits_kernel, grid, dim3(256), 0, st, partial, nsplit, d, rp, r, S);
    return hipGetLastError();
}

// fp32 [d][r] -> bf16 planes [3][rp][d] (hi, mid, lo); columns >= r are zero
__global__ __launch_bounds__(256) void pack_planes_kernel(const float* __restrict__ Q, int64_t d, int r, int rp,
                                                          bf16_t* __restrict__ pack) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= d * rp) return;
    const int64_t row = idx % d;
    const int k = (int)(idx / d);
    const float f = (k < r) ? Q[row * r + k] : 0.f;
    bf16_t hi, mid, lo;
    split3_bf16(f, hi, mid, lo);
    pack[((int64_t)0 * rp + k) * d + row] = hi;
    pack[((int64_t)1 * rp + k) * d + row] = mid;
    pack[((int64_t)2 * rp + k) * d + row] = lo;
}

hipError_t launch_pack_planes(const float* Q, int64_t d, int r, int rp, bf16_t* pack, hipStream_t st) {
    if (d == 0) return hipSuccess;
    dim3 grid((unsigned)((d * rp + 255) / 256));
    hipLaunchKernelGGL(pack_planes_kernel, grid, dim3(256), 0, st, Q, d, r, rp, pack);
    return hipGetLastError();
}

}  // namespace agzo
