// What sits between the linear layers of the gated-MLP stack workload (Alg. 2 over a model): RMS normalisation, the
// SiLU gate and the residual sum.  They are not steps of the method, only the model around it, but a whole-model step
// runs them three times per block, so they are single-pass kernels here: bf16 in and out, fp32 arithmetic, one
// rounding to bf16, 16-byte accesses.  All three are bound by HBM.
#include "agzo_internal.h"

namespace agzo {

__device__ __forceinline__ void unpack8(const uint4& v, float (&f)[8]) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = __uint_as_float(w[i] << 16);
        f[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
}
__device__ __forceinline__ uint4 pack8(const float (&f)[8]) {
    return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
}

// y[t][:] = gain * x[t][:] / sqrt(mean(x[t][:]^2) + eps); one workgroup per row, d a multiple of 8
__global__ __launch_bounds__(256) void glue_rmsnorm_kernel(const bf16_t* __restrict__ x, int64_t ldx, bf16_t* __restrict__ y,
                                                           int64_t ldy, const float* __restrict__ gain, int64_t d, float eps) {
    __shared__ float red[4];
    const int tid = threadIdx.x;
    const bf16_t* xr = x + (int64_t)blockIdx.x * ldx;
    bf16_t* yr = y + (int64_t)blockIdx.x * ldy;
    const int64_t nvec = d / 8;
    float ss = 0.f;
    for (int64_t v = tid; v < nvec; v += 256) {
        float f[8];
        unpack8(*reinterpret_cast<const uint4*>(xr + v * 8), f);
#pragma unroll
        for (int i = 0; i < 8; ++i) ss = fmaf(f[i], f[i], ss);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    const float scale = rsqrtf(((red[0] + red[1]) + (red[2] + red[3])) / (float)d + eps);
    for (int64_t v = tid; v < nvec; v += 256) {          // the row is re-read from cache
        float f[8];
        unpack8(*reinterpret_cast<const uint4*>(xr + v * 8), f);
#pragma unroll
        for (int i = 0; i < 8; ++i) f[i] = f[i] * scale * (gain ? gain[v * 8 + i] : 1.f);
        *reinterpret_cast<uint4*>(yr + v * 8) = pack8(f);
    }
}

// m = silu(a) * u, rows of d (multiple of 8) with leading dimensions
__global__ __launch_bounds__(256) void glue_swiglu_kernel(const bf16_t* __restrict__ a, int64_t lda, const bf16_t* __restrict__ u,
                                                          int64_t ldu, bf16_t* __restrict__ m, int64_t ldm, int64_t n, int64_t d) {
    const int64_t nvec = d / 8;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n * nvec) return;
    const int64_t row = idx / nvec, v = idx - row * nvec;
    float fa[8], fu[8];
    unpack8(*reinterpret_cast<const uint4*>(a + row * lda + v * 8), fa);
    unpack8(*reinterpret_cast<const uint4*>(u + row * ldu + v * 8), fu);
#pragma unroll
    for (int i = 0; i < 8; ++i) fa[i] = fa[i] / (1.f + __expf(-fa[i])) * fu[i];
    *reinterpret_cast<uint4*>(m + row * ldm + v * 8) = pack8(fa);
}

// h += delta (in place)
__global__ __launch_bounds__(256) void glue_add_kernel(bf16_t* __restrict__ h, int64_t ldh, const bf16_t* __restrict__ dl,
                                                       int64_t ldd, int64_t n, int64_t d) {
    const int64_t nvec = d / 8;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n * nvec) return;
    const int64_t row = idx / nvec, v = idx - row * nvec;
    float fh[8], fd[8];
    uint4* ph = reinterpret_cast<uint4*>(h + row * ldh + v * 8);
    unpack8(*ph, fh);
    unpack8(*reinterpret_cast<const uint4*>(dl + row * ldd + v * 8), fd);
#pragma unroll
    for (int i = 0; i < 8; ++i) fh[i] += fd[i];
    *ph = pack8(fh);
}

// ---------------------------------------------------------------------------
// Attention core of a decoder layer (grouped-query, causal, 128-wide heads, per-head RMS normalisation of queries and
// keys, rotary embedding): the model between the q / k / v projections and the o projection.  Two kernels.
//
// prep: q, k <- rope(rmsnorm_per_head(.)), head-major [seq][head][t][128]; v transposed to [seq][kv head][128][t_pad]
//       (t_pad = seq_len rounded up to 32, the padding zero) so that the second product reads keys contiguously.
// attention: one wave = 32 queries of one head (two groups of 16).  Scores are computed transposed, S^T = K Q^T (keys x queries), with
//       v_mfma_f32_16x16x32_bf16: a lane then holds, for ONE query (column lane % 16), the scores of keys 4 g + e of each
//       16-key block (g = lane / 16), so the softmax's running maximum and sum are per-lane scalars up to a reduction
//       over the four g, and the rescaling of the output accumulators (out^T = V^T P^T, same column = query) is a
//       per-lane scalar too.  The eight probabilities a lane holds per 32-key step (two 16-key blocks) go straight into
//       the second product as its operand: a sum over keys does not care about their order, so instead of re-laying P
//       out, V^T is read in the order P is held (keys 4 g .. 4 g + 3 of both blocks: two 8-byte loads).  No LDS.
// ---------------------------------------------------------------------------
constexpr int HEAD_DIM = 128;
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));

// grid.x covers (token, head) pairs of q and k, 16 lanes each; the rotary pair (i, i + 64) sits 8 lanes apart
__global__ __launch_bounds__(256) void glue_qk_prep_kernel(const bf16_t* __restrict__ q, int64_t ldq, const bf16_t* __restrict__ k,
                                                           int64_t ldk, bf16_t* __restrict__ Qr, bf16_t* __restrict__ Kr, int n_seq,
                                                           int seq_len, int n_heads, int n_kv, float log2_theta) {
    const int64_t item = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 4;
    const int j = threadIdx.x & 15;
    const int64_t n_q = (int64_t)n_seq * seq_len * n_heads, n_k = (int64_t)n_seq * seq_len * n_kv;
    if (item >= n_q + n_k) return;                   // whole 16-lane groups leave together
    const bool is_q = item < n_q;
    const int64_t it = is_q ? item : item - n_q;
    const int heads = is_q ? n_heads : n_kv;
    const int64_t tok = it / heads;
    const int head = (int)(it - tok * heads);
    const int seq = (int)(tok / seq_len), t = (int)(tok - (int64_t)seq * seq_len);
    const bf16_t* src = (is_q ? q + tok * ldq : k + tok * ldk) + head * HEAD_DIM + 8 * j;
    float f[8];
    unpack8(*reinterpret_cast<const uint4*>(src), f);
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) ss = fmaf(f[i], f[i], ss);
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) ss += __shfl_xor(ss, off);      // the 16 lanes of this head
    const float scale = rsqrtf(ss / (float)HEAD_DIM + 1e-6f);
    float o[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float mine = f[i] * scale;
        const float other = __shfl_xor(mine, 8);
        const int idx = 8 * (j & 7) + i;                                   // pair index 0..63
        const float inv = exp2f(-(float)idx * (2.0f / HEAD_DIM) * log2_theta);
        float sn, cs;
        sincosf((float)t * inv, &sn, &cs);
        o[i] = (j < 8) ? mine * cs - other * sn : mine * cs + other * sn;  // first half: x1 c - x2 s; second: x2 c + x1 s
    }
    bf16_t* dst = (is_q ? Qr : Kr) + (((int64_t)seq * heads + head) * seq_len + t) * HEAD_DIM + 8 * j;
    *reinterpret_cast<uint4*>(dst) = pack8(o);
}

// Vt[seq][kv head][d][t_pad]: a thread takes 8 values of one token (16-byte load) and stores them to 8 rows; the lanes of
// a wave are consecutive tokens, so every store instruction writes 128 contiguous bytes.  Tokens >= seq_len write zeros.
__global__ __launch_bounds__(256) void glue_v_transpose_kernel(const bf16_t* __restrict__ v, int64_t ldv, bf16_t* __restrict__ Vt,
                                                               int n_seq, int seq_len, int t_pad, int n_kv) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    const int c = blockIdx.y % (HEAD_DIM / 8), head = blockIdx.y / (HEAD_DIM / 8), seq = blockIdx.z;
    if (t >= t_pad) return;
    uint4 raw = make_uint4(0, 0, 0, 0);
    if (t < seq_len) raw = *reinterpret_cast<const uint4*>(v + ((int64_t)seq * seq_len + t) * ldv + head * HEAD_DIM + 8 * c);
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
    bf16_t* dst = Vt + (((int64_t)seq * n_kv + head) * HEAD_DIM + 8 * c) * t_pad + t;
#pragma unroll
    for (int i = 0; i < 8; ++i) dst[(int64_t)i * t_pad] = (bf16_t)((i & 1) ? (w[i >> 1] >> 16) : (w[i >> 1] & 0xFFFFu));
}

// QG 16-query groups per wave: every K and V^T fragment a wave loads serves QG matrix instructions
constexpr int ATT_QG = 2;
constexpr int ATT_WAVE_Q = 16 * ATT_QG;     // queries per wave
constexpr int ATT_WG_Q = 4 * ATT_WAVE_Q;    // queries per workgroup

__global__ __launch_bounds__(256) void glue_attention_kernel(const bf16_t* __restrict__ Qr, const bf16_t* __restrict__ Kr,
                                                             const bf16_t* __restrict__ Vt, bf16_t* __restrict__ out, int64_t ldo,
                                                             int seq_len, int t_pad, int n_heads, int n_kv) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int head = blockIdx.y, seq = blockIdx.z, kvh = head / (n_heads / n_kv);
    // heavy tiles first: the last queries of a sequence see the most keys
    const int q0 = ((int)(gridDim.x - 1 - blockIdx.x) * 4 + wave) * ATT_WAVE_Q;
    if (q0 >= seq_len) return;                                         // wave-uniform
    const bf16_t* Qh = Qr + ((int64_t)seq * n_heads + head) * seq_len * HEAD_DIM;
    const bf16_t* Kh = Kr + ((int64_t)seq * n_kv + kvh) * seq_len * HEAD_DIM;
    const bf16_t* Vh = Vt + ((int64_t)seq * n_kv + kvh) * HEAD_DIM * t_pad;
    union Frag { uint4 u; bf16x8_t v; };
    int qi[ATT_QG];                                                    // rows past the end repeat the last query, unstored
    Frag qf[ATT_QG][4];
#pragma unroll
    for (int qg = 0; qg < ATT_QG; ++qg) {
        qi[qg] = min(q0 + 16 * qg + n, seq_len - 1);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) qf[qg][ks].u = *reinterpret_cast<const uint4*>(Qh + (int64_t)qi[qg] * HEAD_DIM + 32 * ks + 8 * g);
    }
    floatx4_t acc[ATT_QG][8];
#pragma unroll
    for (int qg = 0; qg < ATT_QG; ++qg)
#pragma unroll
        for (int db = 0; db < 8; ++db) acc[qg][db] = floatx4_t{0.f, 0.f, 0.f, 0.f};
    float m_run[ATT_QG], l_run[ATT_QG];
#pragma unroll
    for (int qg = 0; qg < ATT_QG; ++qg) { m_run[qg] = -INFINITY; l_run[qg] = 0.f; }
    const float sc = 1.44269504088896341f * 0.08838834764831845f;      // log2(e) / sqrt(128)
    const int k_end = min(q0 + ATT_WAVE_Q - 1, seq_len - 1);           // last key any query of this wave may see
    // K operand of a 32-key step: this lane's rows are keys kb + 16 blk + n (clamped), its columns 32 ks + 8 g ..
    auto load_k = [&](int kb, Frag (&kf)[2][4]) __attribute__((always_inline)) {
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
            const int krow = min(kb + 16 * blk + n, seq_len - 1);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) kf[blk][ks].u = *reinterpret_cast<const uint4*>(Kh + (int64_t)krow * HEAD_DIM + 32 * ks + 8 * g);
        }
    };
    Frag kf[2][4];
    load_k(0, kf);
    for (int kb = 0; kb <= k_end; kb += 32) {
        // V^T operands of this step: row = dim 16 db + n, the keys in the order the probabilities are held (4 g .. 4 g + 3
        // of both 16-key blocks); requested before the scores so that they arrive under the first product and the softmax
        Frag vf[8];
#pragma unroll
        for (int db = 0; db < 8; ++db) {
            const bf16_t* vrow = Vh + (int64_t)(16 * db + n) * t_pad + kb + 4 * g;
            const uint2 v0 = *reinterpret_cast<const uint2*>(vrow), v1 = *reinterpret_cast<const uint2*>(vrow + 16);
            vf[db].u = make_uint4(v0.x, v0.y, v1.x, v1.y);
        }
        floatx4_t s[ATT_QG][2];
#pragma unroll
        for (int qg = 0; qg < ATT_QG; ++qg)
#pragma unroll
            for (int blk = 0; blk < 2; ++blk) {
                s[qg][blk] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    s[qg][blk] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[blk][ks].v, qf[qg][ks].v, s[qg][blk], 0, 0, 0);
            }
        // the next step's K operands (the step after the last one re-reads clamped rows and is dropped)
        load_k(kb + 32, kf);
#pragma unroll
        for (int qg = 0; qg < ATT_QG; ++qg) {
            // lane: query qi[qg] (column n), keys kb + 16 blk + 4 g + e
            float p[8], mx = m_run[qg];
#pragma unroll
            for (int blk = 0; blk < 2; ++blk)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int key = kb + 16 * blk + 4 * g + e;
                    const float v = (key <= qi[qg] && key < seq_len) ? s[qg][blk][e] * sc : -INFINITY;
                    p[4 * blk + e] = v;
                    mx = fmaxf(mx, v);
                }
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            // a group of queries that sees none of this step's keys (its rows all lie before kb) keeps its state:
            // mx = m_run, alpha = 1, every p = 0.  On a group's first step m_run = -inf and mx is finite (key 0 is visible).
            const float alpha = exp2f(m_run[qg] - mx);
            float psum = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                p[i] = exp2f(p[i] - mx);
                psum += p[i];
            }
            l_run[qg] = l_run[qg] * alpha + psum;
            m_run[qg] = mx;
            Frag pf;
            pf.u = make_uint4(pack_bf16x2(p[0], p[1]), pack_bf16x2(p[2], p[3]), pack_bf16x2(p[4], p[5]), pack_bf16x2(p[6], p[7]));
#pragma unroll
            for (int db = 0; db < 8; ++db) {
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[qg][db][e] *= alpha;
                acc[qg][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[db].v, pf.v, acc[qg][db], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int qg = 0; qg < ATT_QG; ++qg) {
        float l = l_run[qg];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        if (q0 + 16 * qg + n >= seq_len) continue;
        const float inv = 1.f / l;
        bf16_t* orow = out + ((int64_t)seq * seq_len + q0 + 16 * qg + n) * ldo + head * HEAD_DIM + 4 * g;    // dims 16 db + 4 g + e
#pragma unroll
        for (int db = 0; db < 8; ++db)
            *reinterpret_cast<uint2*>(orow + 16 * db) = make_uint2(pack_bf16x2(acc[qg][db][0] * inv, acc[qg][db][1] * inv),
                                                                   pack_bf16x2(acc[qg][db][2] * inv, acc[qg][db][3] * inv));
    }
}

size_t glue_attention_workspace_bytes(int n_seq, int seq_len, int n_heads, int n_kv) {
    const int64_t t_pad = (seq_len + 31) / 32 * 32;
    return (size_t)n_seq * ((int64_t)(n_heads + n_kv) * seq_len + (int64_t)n_kv * t_pad) * HEAD_DIM * sizeof(bf16_t) + 256;
}

hipError_t launch_glue_attention(const bf16_t* q, int64_t ldq, const bf16_t* k, int64_t ldk, const bf16_t* v, int64_t ldv,
                                 bf16_t* out, int64_t ldo, int n_seq, int seq_len, int n_heads, int n_kv, float rope_theta,
                                 void* workspace, hipStream_t st) {
    if (n_seq == 0 || seq_len == 0) return hipSuccess;
    const int t_pad = (seq_len + 31) / 32 * 32;
    bf16_t* Qr = static_cast<bf16_t*>(workspace);
    bf16_t* Kr = Qr + (int64_t)n_seq * n_heads * seq_len * HEAD_DIM;
    bf16_t* Vt = Kr + (int64_t)n_seq * n_kv * seq_len * HEAD_DIM;
    const int64_t items = (int64_t)n_seq * seq_len * (n_heads + n_kv) * 16;
    hipLaunchKernelGGL(glue_qk_prep_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, st, q, ldq, k, ldk, Qr, Kr, n_seq,
                       seq_len, n_heads, n_kv, log2f(rope_theta));
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(glue_v_transpose_kernel, dim3((unsigned)((t_pad + 255) / 256), (unsigned)(n_kv * (HEAD_DIM / 8)), (unsigned)n_seq),
                       dim3(256), 0, st, v, ldv, Vt, n_seq, seq_len, t_pad, n_kv);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(glue_attention_kernel, dim3((unsigned)((seq_len + ATT_WG_Q - 1) / ATT_WG_Q), (unsigned)n_heads, (unsigned)n_seq), dim3(256), 0, st,
                       Qr, Kr, Vt, out, ldo, seq_len, t_pad, n_heads, n_kv);
    return hipGetLastError();
}

hipError_t launch_glue_rmsnorm(const bf16_t* x, int64_t ldx, bf16_t* y, int64_t ldy, const float* gain, int64_t n, int64_t d,
                               float eps, hipStream_t st) {
    if (n == 0 || d == 0) return hipSuccess;
    hipLaunchKernelGGL(glue_rmsnorm_kernel, dim3((unsigned)n), dim3(256), 0, st, x, ldx, y, ldy, gain, d, eps);
    return hipGetLastError();
}

hipError_t launch_glue_swiglu(const bf16_t* a, int64_t lda, const bf16_t* u, int64_t ldu, bf16_t* m, int64_t ldm, int64_t n,
                              int64_t d, hipStream_t st) {
    if (n == 0 || d == 0) return hipSuccess;
    const int64_t items = n * (d / 8);
    hipLaunchKernelGGL(glue_swiglu_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, st, a, lda, u, ldu, m, ldm, n, d);
    return hipGetLastError();
}

hipError_t launch_glue_add(bf16_t* h, int64_t ldh, const bf16_t* dl, int64_t ldd, int64_t n, int64_t d, hipStream_t st) {
    if (n == 0 || d == 0) return hipSuccess;
    const int64_t items = n * (d / 8);
    hipLaunchKernelGGL(glue_add_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, st, h, ldh, dl, ldd, n, d);
    return hipGetLastError();
}

}  // namespace agzo
