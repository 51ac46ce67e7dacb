/*
 * agzo.h - C ABI of the MI355X (gfx950) AGZO hot-path library.
 *
 * One AGZO step for a linear layer (paper Sec. 4.1, Alg. 1, Alg. 2):
 *   sketch the mini-batch activations, orthonormalise to a rank-r basis B,
 *   regenerate the seeded Gaussian factor G, evaluate the loss at
 *   W + eps*G*B^T and W - eps*G*B^T without touching W, form the two-point
 *   scalar g, and apply W -= lr*g*G*B^T in place.
 *
 * Conventions
 *   - Every tensor pointer is DEVICE memory owned by the caller; the library
 *     borrows it until the work enqueued by the call has finished.  Pointers
 *     named *_dev are device scalars/arrays too.  The only host pointers are
 *     the small descriptor structs and the ctx.
 *   - All matrices are row-major.  W is [d_out][d_in] (y = W h, batched
 *     Y = X W^T, Sec. 3.1), X is [n_tokens][d_in] (one token per row: the
 *     transpose of the paper's H), Y is [n_tokens][d_out], the basis B, the
 *     sketches S and the start/iterate Q are [d_in][r] fp32 with leading
 *     dimension r, the projection P is [n_tokens][r] fp32.
 *   - Leading dimensions (ldw, ldx, ldy, ldt) are in elements; for bf16
 *     operands ldw, ldx and d_in must be multiples of 8 and below 2^22, and
 *     W and X must be 16-byte aligned (16-byte rows).
 *   - Calls only enqueue work on the ctx stream (no host synchronisation)
 *     unless stated.  Calls on one ctx must not overlap from several threads.
 *   - Return value: 0 on success, a negative agzo_status otherwise; the text
 *     of the last error is available from agzo_last_error().
 */
#ifndef AGZO_H
#define AGZO_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct agzo_ctx agzo_ctx;

typedef enum {
    AGZO_OK = 0,
    AGZO_EINVAL = -1,   /* null pointer, r < 1, r > 64, r > min(n_tokens, d_in), bad dtype, bad alignment */
    AGZO_ENOMEM = -2,   /* workspace allocation failed */
    AGZO_ENUMERIC = -3, /* Cholesky pivot <= 0: the sketch is rank deficient (reported by agzo_check) */
    AGZO_EHIP = -4      /* HIP runtime error */
} agzo_status;

typedef enum { AGZO_F32 = 0, AGZO_BF16 = 1 } agzo_dtype;
typedef enum { AGZO_LOSS_NONE = 0, AGZO_LOSS_MSE = 1, AGZO_LOSS_CE = 2 } agzo_loss_kind;
typedef enum {
    AGZO_SKETCH_NONE = 0,
    AGZO_SKETCH_RANGE = 1, /* S = X^T Omega, Omega [n_tokens][r] Gaussian from (seed, tag 1): Alg. 1, first product */
    AGZO_SKETCH_POWER = 2, /* S = X^T (X Q) for a given Q [d_in][r]: Alg. 1, power step; Q == NULL: Q is the Gaussian
                              [d_in][r] of (seed, tag 2), the start of the AGZO_INIT_FEATURE variant */
    AGZO_SKETCH_RANGE_FUSED = 3 /* the S of AGZO_SKETCH_RANGE (same Omega; sums in another order), emitted by the forward
                              GEMM itself from the X tiles it stages in LDS instead of by a sweep of its own over X
                              (Sec. 4.1: the f0 pass also yields the subspace information).  Only for bf16 layers whose
                              forward runs in the 128 x 128 tiling (fewer than 160 tiles of 256 x 256, tiling AUTO, W
                              given, squared-error loss or none), r <= 16, n_tokens <= 8192: otherwise AGZO_EINVAL */
} agzo_sketch;

/* Philox stream tags: which Gaussian matrix a (seed, tag, row, col) element belongs to. */
enum { AGZO_TAG_G = 0, AGZO_TAG_OMEGA = 1, AGZO_TAG_Q0 = 2, AGZO_TAG_DENSE = 3 };

enum { AGZO_TILING_AUTO = 0, AGZO_TILING_LARGE = 1 };

/* agzo_step / agzo_basis flags */
enum {
    AGZO_ONE_SIDED = 1,    /* g = (L+ - L0)/eps, the literal form of Eq. 10 / Alg. 2; default is (L+ - L-)/(2 eps) */
    AGZO_NAIVE_INPLACE = 2,/* comparator: perturb W in place, plain forward, undo (Alg. 2's literal schedule); together
                              with AGZO_ONE_SIDED, agzo_step runs Alg. 2 exactly as printed, its last line as one sweep
                              W <- W - (eps + lr g) G B^T over the still-perturbed weights */
    AGZO_INIT_FEATURE = 4, /* start Alg. 1 from a Gaussian Q0 [d_in][r] (tag 2) instead of a token-space Omega */
    AGZO_SHARED_FORWARD = 8/* single layer only: f0, f+ and f- are evaluated from one pass over X and W
                              (Y+- = X W^T +- eps (X B) G^T share the product X W^T); extraction runs first */
};

typedef struct {
    int64_t n_tokens;  /* N = batch x sequence (the paper's m) */
    int64_t d_in;
    int64_t d_out;
    int32_t r;         /* rank of the activation basis, 1..64 */
    int32_t dtype;     /* agzo_dtype of W and X (both the same) */
    int32_t y_dtype;   /* agzo_dtype of Y when stored: F32, or BF16 for bf16 layers */
    int32_t tiling;      /* 0 = the library picks the forward GEMM's tiling from the shape; AGZO_TILING_LARGE = always the
                          * 256 x 256 tiles (tests and measurements; results are the same to rounding order) */
    int64_t ldw, ldx, ldy;
} agzo_layer;

typedef struct {
    int32_t kind;         /* agzo_loss_kind */
    int32_t target_dtype; /* MSE: AGZO_F32 or AGZO_BF16 target values; ignored for CE */
    const void* target;   /* MSE: Y* [n_tokens][d_out], ld = ldt.  CE: int32 ids [n_tokens] in [0, d_out), < 0 = ignored row
                             (loss = mean over the other rows of -log softmax(Y[row])[id], natural log); an id >= d_out
                             is a caller error that the kernels survive: such a row is skipped like an ignored one */
    int64_t ldt;
} agzo_loss_spec;

/* Create a context that enqueues on hip_stream (a hipStream_t, borrowed; NULL = default stream)
 * of the current device.  The ctx owns a workspace that grows on demand (growth synchronises). */
int agzo_create(agzo_ctx** out, void* hip_stream);
void agzo_destroy(agzo_ctx* ctx);
const char* agzo_last_error(const agzo_ctx* ctx);
/* Synchronise the stream and report a deferred numeric failure (AGZO_ENUMERIC) if any; clears it. */
int agzo_check(agzo_ctx* ctx);

/* Measurement hooks (no counterpart in the paper): each launch of a selected kernel class is bracketed
 * by HIP events recorded on the ctx stream; agzo_profile_read synchronises and returns the number of
 * launches since agzo_profile_enable and the sum of their durations in milliseconds.
 * mask: bit (1 << AGZO_PROF_x) selects class x, AGZO_PROF_ALL all of them, 0 switches timing off.  The events
 * cost a few microseconds of stream time each, so a timed region should select only what it reports. */
enum { AGZO_PROF_GEMM = 0, AGZO_PROF_UPDATE = 1, AGZO_PROF_XQ = 2, AGZO_PROF_XTT = 3, AGZO_PROF_QR = 4,
       AGZO_PROF_FILL = 5, AGZO_PROF_KINDS = 6, AGZO_PROF_ALL = 63 };
int agzo_profile_enable(agzo_ctx* ctx, int32_t mask);
int agzo_profile_read(agzo_ctx* ctx, int32_t kind, int64_t* launches, double* total_ms);
/* Shader clock during the GEMM class (no counterpart in the paper): while AGZO_PROF_GEMM is selected, the first
 * workgroup of every bf16 GEMM launch (up to 8192 launches per agzo_profile_enable) records the GPU's shader-clock
 * counter and its constant-rate counter at entry and exit.  Synchronises; *launches = records taken, *mean_ghz =
 * sum of shader cycles / sum of elapsed time over them (0 if none).  Both outputs are host pointers. */
int agzo_profile_clock(agzo_ctx* ctx, int64_t* launches, double* mean_ghz);
/* Device probe (no counterpart in the paper; a yardstick for the measured MFMA roofline fraction): one workgroup of
 * four waves per compute unit runs `iters` iterations of 8 groups of 16 v_mfma_f32_32x32x16_bf16 on register
 * operands only (no LDS, no memory traffic inside the loop); `duty` (1..8) of every 8 groups are issued, the rest
 * replaced by a sleep of similar length; duty = 9 issues the flop count of all 8 groups as 256
 * v_mfma_f32_16x16x32_bf16 over 64 accumulators of four accumulation registers.  operands: device, 32 KiB of bf16 bit patterns, read as 8 x 256 16-byte
 * vectors (vector i*256 + t feeds lane t: i < 4 A fragments, i >= 4 B fragments); how often these bits toggle decides
 * the power drawn and with it the clock the device holds.  Synchronous: enqueues on the ctx stream, waits, and
 * returns the matrix rate over workgroup 0's lifetime in *tflops and the mean shader clock in *clock_ghz (host
 * pointers).  Errors: AGZO_EINVAL for NULL pointers or duty (1..9) / iters (1..2^20) out of range. */
int agzo_probe_mfma(agzo_ctx* ctx, const void* operands, int32_t duty, int32_t iters, double* tflops, double* clock_ghz);

/* Generator (Alg. 2 "generate R from seed"; this build: Philox4x32-10 + Box-Muller).
 * words: uint32 [rows][cols], word (row, col) = word col%4 of Philox(counter (row, col/4, tag, 0),
 * key (seed lo, seed hi)).  normal: fp32 [rows][cols] from the same words, u = ((x>>9)+0.5)*2^-23,
 * (z0,z1) = sqrt(-2 ln u0) (cos, sin)(2 pi u1), (z2,z3) likewise. */
int agzo_philox_words(agzo_ctx* ctx, uint32_t* dst, int64_t rows, int32_t cols, uint64_t seed, uint32_t tag);
int agzo_fill_normal(agzo_ctx* ctx, float* dst, int64_t rows, int32_t cols, uint64_t seed, uint32_t tag);

/* Base forward (f0 of Sec. 4.1) with sketch emission (Alg. 1 products):
 *   Y = X W^T (stored if Y != NULL), loss -> *loss_dev (if loss && loss_dev),
 *   S = X^T Omega (RANGE) or X^T (X Q) (POWER) -> S [d_in][r].
 * W may be NULL together with Y == NULL and no loss: sketch only. */
int agzo_layer_forward_sketch(agzo_ctx* ctx, const agzo_layer* L, const void* W, const void* X, void* Y,
                              int32_t mode, const float* Q, uint64_t seed, float* S,
                              const agzo_loss_spec* loss, double* loss_dev);

/* Thin QR with positive diagonal of a tall fp32 matrix S [d_in][r] -> Q [d_in][r]
 * (the "qr" steps of Alg. 1; CholeskyQR2 with fp64 Gram and Cholesky). */
int agzo_qr(agzo_ctx* ctx, const float* S, int64_t d_in, int32_t r, float* Q);

/* Alg. 1 SubspaceExtract: B = orthonormal basis after K power steps.  S0, if not NULL, is the
 * first sketch already produced by agzo_layer_forward_sketch(RANGE) with the same seed. */
int agzo_basis(agzo_ctx* ctx, const agzo_layer* L, const void* X, int32_t K, uint64_t seed,
               const float* S0, int32_t flags, float* B);

/* Alg. 1 for n layers at once (Alg. 2, first loop: the base forward computes every layer's basis; the extractions are
 * independent of each other).  Per item the arguments of agzo_basis; every stage of the algorithm (test matrix,
 * sketches, orthonormalisations, power steps) is one launch for up to 16 bf16 layers whose ranks round up to the same
 * multiple of 16, instead of one per layer, which is what a set of small layers is bound by.  Every B is bit-identical
 * to what agzo_basis gives for the same item.  items: host array, read during the call only; the B of different items
 * must not overlap.  n = 0 is a no-op.  Errors: AGZO_EINVAL for n < 0, NULL items, or an item agzo_basis would reject
 * (nothing is enqueued then). */
typedef struct {
    agzo_layer layer;   /* d_out, ldw, ldy, y_dtype are not used */
    const void* X;
    uint64_t seed;
    const float* S0;    /* nullable, as for agzo_basis */
    float* B;           /* [d_in][r] out */
} agzo_basis_item;
int agzo_basis_many(agzo_ctx* ctx, const agzo_basis_item* items, int32_t n, int32_t K, int32_t flags);

/* Perturbed forward (f+ / f- of Sec. 4.1, Eq. 7): Y = X W^T + eps_signed (X B) G^T with G [d_out][r]
 * regenerated from (seed, tag 0); W is not modified.  Loss as above. */
int agzo_perturbed_forward(agzo_ctx* ctx, const agzo_layer* L, const void* W, const void* X,
                           const float* B, uint64_t seed, float eps_signed, void* Y,
                           const agzo_loss_spec* loss, double* loss_dev);

/* Projected-gradient scalar (Eq. 10, Alg. 2): out4_dev = {L0, L+, L-, g} (device doubles); reads the losses and writes
 * g = (L+ - L-) / (2 eps), or with AGZO_ONE_SIDED the paper's literal g = (L+ - L0) / eps (L- is then set to 0).
 * For schedules that the caller composes from the calls above (several layers sharing one global g): every layer's
 * agzo_update can take out4_dev + 3 as its g_dev.  Errors: AGZO_EINVAL for NULL or eps <= 0. */
int agzo_two_point(agzo_ctx* ctx, double* out4_dev, float eps, int32_t flags);

/* In-place rank-r sweep (Alg. 2, restore/update line): W -= lr * g * G B^T, g = *g_dev (1 if NULL). */
int agzo_update(agzo_ctx* ctx, const agzo_layer* L, void* W, const float* B, uint64_t seed,
                float lr, const double* g_dev);

/* agzo_update for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical results; the scratch that a bf16
 * update needs (both factors as bf16 hi/lo matrix-core fragments: 4 r16 (d_out rounded up to 32 + d_in rounded up to
 * 256) bytes, r16 = r rounded up to 16; 1 MiB for a 12288 x 4096 matrix at r = 16) lives in a static device array of 8 MiB that each GPU the library runs on holds until
 * the process ends, instead of the context's growable workspace.  The call allocates and frees nothing.  fp32
 * matrices need no scratch.  Every call on a GPU shares that GPU's array (also across contexts): calls that may
 * overlap on one GPU (different streams) race and must be ordered by the caller; nothing in the array has to start
 * at zero, every call rewrites all of what it reads.  The device current at the call must be the one the context was
 * created on.  Errors: as agzo_update; AGZO_EINVAL when the fragments exceed the 8 MiB or the device differs
 * (nothing is enqueued then). */
int agzo_update_noalloc(agzo_ctx* ctx, const agzo_layer* L, void* W, const float* B, uint64_t seed,
                        float lr, const double* g_dev);

/* The same sweep for n matrices at once (Alg. 2: every layer is updated after the one scalar g is known, so the
 * updates of a model arrive together).  items: host array, read during the call only; per item the arguments of
 * agzo_update: W device [d_out][ldw] of `dtype`, B device fp32 [d_in][r], g_dev device scalar or NULL (= 1), seed of
 * that layer's Gaussian factor, lr; reserved must be 0.  bf16 matrices whose ranks round up to the same multiple of 16
 * share one preparation launch and one sweep per 16 matrices (small matrices no longer pay two launches each); fp32
 * matrices are swept one by one.  Every matrix ends bit-identical to what agzo_update gives it.  The matrices must
 * not overlap.  n = 0 is a no-op.  Errors: AGZO_EINVAL for n < 0, NULL items, or an item agzo_update would reject
 * (nothing is enqueued then). */
typedef struct {
    void* W;
    const float* B;
    const double* g_dev;
    int64_t d_out, d_in, ldw;
    int32_t r;
    int32_t dtype;     /* agzo_dtype of W */
    uint64_t seed;
    float lr;
    int32_t reserved;
} agzo_update_item;
int agzo_update_many(agzo_ctx* ctx, const agzo_update_item* items, int32_t n);

/* Dense Gaussian sweep for parameters that are not linear-layer weights (Eq. 7, second branch; Alg. 2: the perturb,
 * restore and update lines for such parameters): theta[i][j] += coef * z(i, j) in place, z the N(0,1) value
 * (seed, tag 3, row i, column j) of the generator above, coef = scale * *g_dev (scale alone if g_dev is NULL).
 * theta: device, [rows][cols] with row stride ld elements, dtype AGZO_F32 or AGZO_BF16 (fp32 arithmetic, one rounding
 * to the storage type; bf16 to nearest even).  A vector of n parameters is rows = 1, cols = n or any other fixed
 * factorisation: the perturbation, its reversal and the update must use the same one.  Perturb with scale = +eps,
 * go to the other side with -2 eps, restore with +eps, update with scale = -lr and g_dev = the scalar of
 * agzo_two_point.  Errors: AGZO_EINVAL for NULL theta, negative sizes, ld < cols, rows or cols/4 >= 2^32, bad dtype. */
int agzo_dense_perturb(agzo_ctx* ctx, void* theta, int32_t dtype, int64_t rows, int64_t cols, int64_t ld, uint64_t seed,
                       float scale, const double* g_dev);

/* One whole AGZO step for one layer (Alg. 2).  out_dev[4] = {L0, L+, L-, g} (device doubles). */
int agzo_step(agzo_ctx* ctx, const agzo_layer* L, void* W, const void* X, const agzo_loss_spec* loss,
              int32_t K, float eps, float lr, uint64_t seed, int32_t flags, double* out_dev);

/* The same step without its last line (Alg. 2 up to and including g): out_dev as above, the basis goes to
 * B_out (device fp32 [d_in][r], required) and W is left unchanged, for callers that update several layers together
 * with agzo_update_many (g_dev = out_dev + 3, or a scalar of their own).  Flags as for agzo_step; with
 * AGZO_NAIVE_INPLACE W is perturbed and restored inside the call.  Errors as agzo_step, AGZO_EINVAL for NULL B_out. */
int agzo_step_no_update(agzo_ctx* ctx, const agzo_layer* L, void* W, const void* X, const agzo_loss_spec* loss,
                        int32_t K, float eps, uint64_t seed, int32_t flags, double* out_dev, float* B_out);

/* The model around the linear layers of a gated-MLP stack (not steps of the method; a whole-model step of Alg. 2 runs
 * them once per block and pass, so they are single-pass kernels): bf16 device tensors of n rows of d values (d a
 * multiple of 8, 16-byte aligned rows, leading dimensions in elements), fp32 arithmetic, one rounding to bf16.
 *   rmsnorm: y[t] = gain * x[t] / sqrt(mean(x[t]^2) + eps)   (gain: device fp32 [d], NULL = 1; y may alias x)
 *   swiglu : m = silu(a) * u, silu(z) = z / (1 + exp(-z))     (m may alias a or u)
 *   add    : h += delta in place
 *   attention: the core of a decoder layer between its q / k / v projections and its o projection: grouped-query causal
 *            attention with 128-wide heads, queries and keys RMS-normalised per head (gain 1, eps 1e-6) and rotated by
 *            the rotary embedding (pairs (i, i + 64) of a head by the angle t rope_theta^(-2i/128), t the position inside
 *            the sequence), scores scaled by 1/sqrt(128), softmax in fp32, probabilities rounded to bf16 for the second
 *            product.  q [N][n_heads 128], k and v [N][n_kv_heads 128], out [N][n_heads 128], N = n_seq seq_len tokens,
 *            the sequences back to back; n_heads a multiple of n_kv_heads.  Uses (and may grow) the context's workspace.
 * Errors: AGZO_EINVAL for NULL or misaligned tensors, d % 8 != 0, leading dimensions below d, a bad attention shape. */
int agzo_glue_attention(agzo_ctx* ctx, const void* q, int64_t ldq, const void* k, int64_t ldk, const void* v, int64_t ldv,
                        void* out, int64_t ldo, int32_t n_seq, int32_t seq_len, int32_t n_heads, int32_t n_kv_heads,
                        float rope_theta);
int agzo_glue_rmsnorm(agzo_ctx* ctx, const void* x, int64_t ldx, void* y, int64_t ldy, const float* gain, int64_t n, int64_t d,
                      float eps);
int agzo_glue_swiglu(agzo_ctx* ctx, const void* a, int64_t lda, const void* u, int64_t ldu, void* m, int64_t ldm, int64_t n,
                     int64_t d);
int agzo_glue_add(agzo_ctx* ctx, void* h, int64_t ldh, const void* delta, int64_t ldd, int64_t n, int64_t d);

/* Alg. 2 for n independent single-layer problems in one call (a layer set whose projections each have their own loss
 * and their own scalar g): every layer's base forward, all bases together (as agzo_basis_many), all projections X B
 * in one launch, the perturbed forwards, every scalar, and all updates in one batched sweep (as agzo_update_many).
 * Per item the arguments of agzo_step; out_dev[4] = {L0, L+, L-, g} per item.  B_out != NULL: that item's basis goes
 * there and its W is left unchanged (as agzo_step_no_update).  Results per item are bit-identical to agzo_step with the
 * same arguments.  Flags: AGZO_ONE_SIDED, AGZO_INIT_FEATURE, AGZO_SHARED_FORWARD; AGZO_NAIVE_INPLACE is refused.
 * Errors: AGZO_EINVAL for a bad list or an item agzo_step would reject (nothing is enqueued then). */
typedef struct {
    agzo_layer layer;
    void* W;
    const void* X;
    agzo_loss_spec loss;
    uint64_t seed;
    double* out_dev;
    float* B_out;       /* nullable */
} agzo_step_item;
int agzo_step_many(agzo_ctx* ctx, const agzo_step_item* items, int32_t n, int32_t K, float eps, float lr, int32_t flags);

#ifdef __cplusplus
}
#endif
#endif /* AGZO_H */
