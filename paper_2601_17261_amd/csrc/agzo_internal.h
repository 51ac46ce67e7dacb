// Internal declarations shared by the HIP sources of libagzo (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "agzo.h"

namespace agzo {

constexpr int kMaxRank = 64;

// ---------------------------------------------------------------------------
// bf16 helpers (bit-level; bf16 = upper half of an fp32)
// ---------------------------------------------------------------------------
typedef uint16_t bf16_t;

__device__ __forceinline__ float bf16_to_f32(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// round to nearest, ties to even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    const __bf16 b = (__bf16)f;
    return __builtin_bit_cast(bf16_t, b);
}

// two values rounded and packed: a in the low half, b in the high half
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const f32x2 v = {a, b};
    const bf16x2 h = __builtin_convertvector(v, bf16x2);
    return __builtin_bit_cast(uint32_t, h);
}

// f = hi + mid + lo with each part a bf16: 24 significant bits in total, so the
// three-term sum reproduces an fp32 value exactly (up to the bf16 exponent range).
__device__ __forceinline__ void split3_bf16(float f, bf16_t& hi, bf16_t& mid, bf16_t& lo) {
    hi = f32_to_bf16(f);
    float r1 = f - bf16_to_f32(hi);
    mid = f32_to_bf16(r1);
    float r2 = r1 - bf16_to_f32(mid);
    lo = f32_to_bf16(r2);
}

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11) and the Box-Muller map used for every
// Gaussian matrix of the method (Alg. 2: generated from a seed, never stored).
// counter = (row, col/4, tag, 0), key = (seed lo, seed hi).
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1) {
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int i = 0; i < 10; ++i) {
        uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
        uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
        uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += W0; k1 += W1;
    }
    return make_uint4(c0, c1, c2, c3);
}

__device__ __forceinline__ float philox_uniform(uint32_t x) {
    // 23 random bits plus a half: exact in fp32, strictly inside (0, 1)
    return ((float)(x >> 9) + 0.5f) * 1.1920928955078125e-07f;  // 2^-23
}

__device__ __forceinline__ void box_muller(uint32_t xa, uint32_t xb, float& z0, float& z1) {
    float rad = sqrtf(-2.0f * logf(philox_uniform(xa)));
    float s, c;
    sincospif(2.0f * philox_uniform(xb), &s, &c);
    z0 = rad * c;
    z1 = rad * s;
}

// four normals for columns 4*quad .. 4*quad+3 of `row`
__device__ __forceinline__ float4 philox_normal4(uint32_t seed_lo, uint32_t seed_hi, uint32_t tag,
                                                 uint32_t row, uint32_t quad) {
    uint4 x = philox4x32_10(row, quad, tag, 0u, seed_lo, seed_hi);
    float4 z;
    box_muller(x.x, x.y, z.x, z.y);
    box_muller(x.z, x.w, z.z, z.w);
    return z;
}

// ---------------------------------------------------------------------------
// Several independent problems in one launch (the extractions of a model's layers, Alg. 2 first loop): the argument
// sets travel as a kernel argument, a workgroup finds its problem from the running workgroup counts (uniform: a few
// scalar compares) and then runs exactly the code of the single-problem kernel, so results are bit-identical.
// ---------------------------------------------------------------------------
constexpr int kBatchMax = 16;
template <typename A>
struct KBatch {
    int n;
    uint32_t first[kBatchMax];   // first workgroup of problem m
    uint32_t gx[kBatchMax];      // its grid width (workgroups along x); y = local / gx
    A a[kBatchMax];
};
// index of the problem that workgroup blockIdx.x belongs to; bx, by: its coordinates inside that problem's grid
template <typename A>
__device__ __forceinline__ int kbatch_find(const KBatch<A>& tb, uint32_t& bx, uint32_t& by) {
    int m = 0;
    while (m + 1 < tb.n && blockIdx.x >= tb.first[m + 1]) ++m;
    const uint32_t local = blockIdx.x - tb.first[m];
    by = local / tb.gx[m];
    bx = local - by * tb.gx[m];
    return m;
}

// ---------------------------------------------------------------------------
// host-side launch functions (one per source file); all enqueue on `st`
// ---------------------------------------------------------------------------
struct GemmLossArgs {
    int kind;             // agzo_loss_kind
    int target_dtype;     // agzo_dtype
    const void* target;
    int64_t ldt;
    double* partials;     // [n_workgroups] (MSE) scratch
    // cross-entropy scratch: (max, sum exp) per (phase, column chunk, token) and target logit per (phase, token)
    void* ce_ms = nullptr;
    float* ce_tl = nullptr;
};

// philox.hip
hipError_t launch_philox_words(uint32_t* dst, int64_t rows, int cols, uint64_t seed, uint32_t tag, hipStream_t st);
hipError_t launch_fill_normal(float* dst, int64_t rows, int cols, uint64_t seed, uint32_t tag, hipStream_t st);
// bf16 [3][rp][n_pad] hi/mid/lo planes of Omega^T (rows of Omega are tokens)
hipError_t launch_fill_normal_packT(bf16_t* dst, int64_t n, int64_t n_pad, int r, int rp, uint64_t seed,
                                    uint32_t tag, hipStream_t st);

struct FillPackTArgs { bf16_t* dst; int64_t n, n_pad; int r, rp; uint64_t seed; uint32_t tag; };
// the same for up to kBatchMax matrices in one launch
hipError_t launch_fill_normal_packT_many(const FillPackTArgs* a, int n, hipStream_t st);

// gemm_bf16.hip : Y = X W^T (+ P' G^T), MFMA, fused loss partials
struct GemmBf16Args {
    const bf16_t* X; int64_t ldx;
    const bf16_t* W; int64_t ldw;
    int64_t M, N, K;            // tokens, d_out, d_in
    void* Y; int y_dtype; int64_t ldy;
    const float* P; int r;      // projection X B [M][r] (NULL: no rank-r term)
    float eps_signed; uint64_t seed;
    GemmLossArgs loss;
    // shared = true: one pass evaluates the loss at W, W + eps Z and W - eps Z (eps = eps_signed > 0);
    // the loss partials are then [3][n_workgroups] and Y must be NULL
    bool shared = false;
    // true: always the 256 x 256 tiling (default: shapes with few such tiles take the 128 x 128 one when the call is
    // one it supports); must agree with the small_ok given to gemm_bf16_num_workgroups when the workspace was sized
    bool large_tiles = false;
    // gemm_bf16_ext_bytes() bytes of device scratch for the rank-r extension operands of a perturbed forward
    // (NULL: every tile builds them itself)
    void* ext_ws = nullptr;
    // fused range sketch S = X^T Omega (NULL: none; only where gemm_bf16_fuses_sketch() says so): Omega^T as bf16
    // planes [3][16][sk_mpad], sk_mpad = gemm_bf16_sketch_mpad(M); sk_partial receives gemm_bf16_sketch_splits(M)
    // partial sums [split][K][16], one per 128-token tile
    const bf16_t* sk_T = nullptr; int64_t sk_mpad = 0; float* sk_partial = nullptr;
    // telemetry (NULL: none): four 64-bit device words that workgroup 0 fills with the shader-clock counter and the
    // constant-rate counter at kernel entry and exit
    unsigned long long* clk = nullptr;
};
// number of loss partials a launch writes; small_ok: the call is one the 128 x 128 tiling supports (no shared-forward
// mode, no cross-entropy), which is then used for shapes with few 256 x 256 tiles
int gemm_bf16_num_workgroups(int64_t M, int64_t N, bool small_ok);
size_t gemm_bf16_ext_bytes(int64_t M, int64_t N, int r);
// true: a plain forward of this shape (no rank-r term, no shared-forward mode, no cross-entropy) runs in the 128 x 128
// tiling, whose kernel can emit the range sketch from its LDS-staged X tiles (r <= 16, at most 64 token tiles)
bool gemm_bf16_fuses_sketch(int64_t M, int64_t N, int r, bool large_tiles);
inline int64_t gemm_bf16_sketch_mpad(int64_t M) { return (M + 127) / 128 * 128; }
inline int gemm_bf16_sketch_splits(int64_t M) { return (int)((M + 127) / 128); }
hipError_t launch_gemm_bf16(const GemmBf16Args& a, hipStream_t st);

// gemm_f32.hip : generic strided fp32 GEMM with fp64 accumulation, and the fp32 epilogue
hipError_t launch_gemm_f32(const float* A, int64_t sam, int64_t sak, const float* B, int64_t sbk, int64_t sbn,
                           float* C, int64_t ldc, int64_t M, int64_t N, int64_t K, hipStream_t st);
int epilogue_f32_num_workgroups(int64_t M, int64_t N);
// Y[t][j] += eps_signed * sum_k P[t][k] G[j][k] (if P), then loss partials (if loss.kind)
hipError_t launch_epilogue_f32(float* Y, int64_t ldy, int64_t M, int64_t N, const float* P, int r,
                               float eps_signed, uint64_t seed, const GemmLossArgs& loss, hipStream_t st);

// skinny.hip : bf16 tall-skinny products
// T = X Qp, Qp given as bf16 planes [3][rp][d_in]; writes T fp32 [M][r] (nullable) and
// T^T planes bf16 [3][rp][m_pad] (nullable)
// part: xq_part_bytes() bytes of scratch for the split over d_in that small token counts take (NULL: never split)
size_t xq_part_bytes(int64_t M, int64_t K, int rp);
hipError_t launch_xq_bf16(const bf16_t* X, int64_t ldx, int64_t M, int64_t K, const bf16_t* Qpack, int r, int rp,
                          float* T, bf16_t* TpackT, int64_t m_pad, float* part, hipStream_t st);
struct XqArgs { const bf16_t* X; int64_t ldx, M, K; const bf16_t* Qpack; int r, rp; float* T; bf16_t* TpackT; int64_t m_pad; float* part; };
// up to kBatchMax products with the same rp in one launch (plus one finishing launch if any of them splits d_in)
hipError_t launch_xq_bf16_many(const XqArgs* a, int n, hipStream_t st);
int xtt_num_splits(int64_t M, int64_t K);
// partial[s][d][rp] = sum over token range s of X[t][d] * T[t][k]
hipError_t launch_xtt_bf16(const bf16_t* X, int64_t ldx, int64_t M, int64_t K, const bf16_t* TpackT, int64_t m_pad,
                           int rp, float* partial, int nsplit, hipStream_t st);
struct XttArgs { const bf16_t* X; int64_t ldx, M, K; const bf16_t* TpackT; int64_t m_pad; int rp; float* partial; int nsplit; };
hipError_t launch_xtt_bf16_many(const XttArgs* a, int n, hipStream_t st);
hipError_t launch_reduce_splits(const float* partial, int nsplit, int64_t d, int rp, int r, float* S, hipStream_t st);
// Q fp32 [d][r] -> bf16 planes [3][rp][d]
hipError_t launch_pack_planes(const float* Q, int64_t d, int r, int rp, bf16_t* pack, hipStream_t st);

// qr.hip : CholeskyQR2
size_t qr_workspace_bytes(int64_t d, int r);
// S explicit, or splits [nsplit][d][rp] (then their fp32 sum is also stored to S_out); Q fp32 out;
// planes (nullable) bf16 [3][rp][d]; refine = false: single Cholesky pass (for iterates that are sketched again)
hipError_t launch_qr(const float* S, const float* splits, int nsplit, int rp, float* S_out, int64_t d, int r, float* Q,
                     bf16_t* planes, void* workspace, int* numeric_flag, bool refine, hipStream_t st);

struct QrArgs { const float* S; const float* splits; int nsplit; int rp; float* S_out; int64_t d; int r; float* Q; bf16_t* planes; void* workspace; };
// up to kBatchMax factorisations with the same rp, each launch of the sequence serving all of them
hipError_t launch_qr_many(const QrArgs* a, int n, int* numeric_flag, bool refine, hipStream_t st);

// update.hip : W -= (lr * g + shift) * G B^T in place, g = *g_dev (1 if NULL)
// workspace: update_workspace_bytes() bytes of device scratch (may be NULL when that is 0)
size_t update_workspace_bytes(int dtype, int64_t d_out, int64_t d_in, int r);
hipError_t launch_update(void* W, int dtype, int64_t ldw, int64_t d_out, int64_t d_in, const float* B, int r,
                         uint64_t seed, float lr, const double* g_dev, void* workspace, hipStream_t st,
                         float shift = 0.f);
// the same for n bf16 matrices that share nk = ceil(r / 16), n <= update_many_max(), in two launches; the workspace
// holds the sum of their update_workspace_bytes()
struct UpdateDesc {
    void* W;
    const float* B;
    const double* g_dev;
    int64_t ldw, d_out, d_in;
    uint64_t seed;
    float lr;
    int r;
};
int update_many_max();
// bf16 matrices with r = 1 (at most kBatchMax): one launch, no scratch
hipError_t launch_update_rank1_many(const UpdateDesc* d, int n, hipStream_t st);
hipError_t launch_update_many(const UpdateDesc* d, int n, int nk, void* workspace, hipStream_t st);

// loss.hip
// cross-entropy from the GEMM's per-chunk softmax statistics: out[ph] = mean over rows with target >= 0 of
// log(sum exp) - logit[target];  ms: float2 [nphase][nchunk][M], tl: float [nphase][M]
int gemm_bf16_ce_chunks(int64_t N);
hipError_t launch_ce_combine(const void* ms, const float* tl, const int32_t* target, int64_t M, int64_t N, int nchunk,
                             int nphase, double* scratch, double* out, hipStream_t st);
// cross-entropy of stored fp32 logits Y [M][N] (fp32-storage path): out[0] as above
hipError_t launch_ce_rows_f32(const float* Y, int64_t ldy, int64_t M, int64_t N, const int32_t* target, double* scratch,
                              double* out, hipStream_t st);
// out[b] = scale * sum(partials[b*n .. b*n+n)), b < nout
hipError_t launch_finish_loss(const double* partials, int n, double scale, double* out, int nout, hipStream_t st);
hipError_t launch_two_point(double* out4, float eps, int one_sided, hipStream_t st);
// both in one launch: partials [nphase][n] (phase 0 = f0, 1 = f+, 2 = f-; nphase = 2 for the one-sided form) -> out4
hipError_t launch_finish_two_point(const double* partials, int n, double scale, int nphase, double* out4, float eps,
                                   int one_sided, hipStream_t st);

// update.hip : theta[i][j] += scale * (*g_dev or 1) * z(i, j), z = Philox normal of stream AGZO_TAG_DENSE (rows < 2^32)
hipError_t launch_dense_axpy(void* theta, int dtype, int64_t rows, int64_t cols, int64_t ld, uint64_t seed, float scale,
                             const double* g_dev, hipStream_t st);

// glue.hip : the model around the linear layers of the MLP-stack workload (bf16 rows of d, d % 8 == 0, 16-byte aligned)
hipError_t launch_glue_rmsnorm(const bf16_t* x, int64_t ldx, bf16_t* y, int64_t ldy, const float* gain, int64_t n, int64_t d,
                               float eps, hipStream_t st);
hipError_t launch_glue_swiglu(const bf16_t* a, int64_t lda, const bf16_t* u, int64_t ldu, bf16_t* m, int64_t ldm, int64_t n,
                              int64_t d, hipStream_t st);
hipError_t launch_glue_add(bf16_t* h, int64_t ldh, const bf16_t* dl, int64_t ldd, int64_t n, int64_t d, hipStream_t st);

// attention core of a decoder layer (128-wide heads): q [N][n_heads 128], k, v [N][n_kv 128] bf16, N = n_seq seq_len tokens,
// sequences back to back -> out [N][n_heads 128]; workspace: glue_attention_workspace_bytes() of device scratch
size_t glue_attention_workspace_bytes(int n_seq, int seq_len, int n_heads, int n_kv);
hipError_t launch_glue_attention(const bf16_t* q, int64_t ldq, const bf16_t* k, int64_t ldk, const bf16_t* v, int64_t ldv,
                                 bf16_t* out, int64_t ldo, int n_seq, int seq_len, int n_heads, int n_kv, float rope_theta,
                                 void* workspace, hipStream_t st);

// probe.hip : register-only MFMA loop for measuring the sustained matrix rate and shader clock of the device;
// clk4: four 64-bit words for the counters plus 1 KiB that the kernel may (never does) write behind them
hipError_t launch_probe_mfma(const void* operands, int duty, int iters, unsigned long long* clk4, hipStream_t st);

}  // namespace agzo
