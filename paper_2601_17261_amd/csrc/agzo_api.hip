// C ABI of libagzo: argument checks, workspace carving and the stream-ordered sequence of kernel
// launches that makes up one AGZO step (Alg. 2) for a linear layer.  No arithmetic lives here.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <initializer_list>
#include <mutex>
#include <new>
#include <vector>

#include "agzo_internal.h"

using namespace agzo;

struct ProfClass {
    std::vector<hipEvent_t> start, stop;
    size_t used = 0;
};

// Scratch of agzo_update_noalloc: the factor fragments of one bf16 update, for callers that cannot allocate.
// One copy per GPU, held until the process ends; its device address is resolved once per device (resolve_scratch).
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

struct agzo_ctx {
    hipStream_t stream;
    int device;            // the device that was current at agzo_create
    char* static_scratch;  // device address of `scratch` on that device
    char err[512];
    char* ws;
    size_t ws_bytes;
    int* flag;   // device int: deferred numeric failure
    uint32_t prof;      // mask of timed kernel classes (bit = AGZO_PROF_* value)
    ProfClass pc[AGZO_PROF_KINDS];
    // clock telemetry: kClkSlots records of four 64-bit words (one per timed GEMM launch), then the probe's record
    unsigned long long* clk;
    size_t clk_used;
};
constexpr size_t kClkSlots = 8192;
constexpr size_t kClkBytes = (kClkSlots + 1) * 32 + 1024;

namespace {

int fail(agzo_ctx* c, int code, const char* fmt, ...) {
    if (c) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(c->err, sizeof(c->err), fmt, ap);
        va_end(ap);
    }
    return code;
}

#define HIPCHK(expr)                                                                              \
    do {                                                                                          \
        hipError_t e__ = (expr);                                                                  \
        if (e__ != hipSuccess) return fail(ctx, AGZO_EHIP, "%s: %s", #expr, hipGetErrorString(e__)); \
    } while (0)
#define TRY(expr)              \
    do {                       \
        int rc__ = (expr);     \
        if (rc__ != 0) return rc__; \
    } while (0)

// Optional timing of one kernel class with HIP events recorded on the ctx stream around each launch.
struct ProfScope {
    agzo_ctx* c;
    int kind;
    hipEvent_t stop = nullptr;
    ProfScope(agzo_ctx* ctx, int k) : c(ctx), kind(k) {
        if (!((c->prof >> kind) & 1u)) return;
        ProfClass& pc = c->pc[kind];
        if (pc.used == pc.start.size()) {
            hipEvent_t a, b;
            if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return;
            pc.start.push_back(a);
            pc.stop.push_back(b);
        }
        (void)hipEventRecord(pc.start[pc.used], c->stream);
        stop = pc.stop[pc.used];
        pc.used++;
    }
    ~ProfScope() {
        if (stop) (void)hipEventRecord(stop, c->stream);
    }
};

// Device address of the static scratch array on the current device.  The array's name is only a host-side handle
// for the symbol: every use of its memory goes through the address looked up here, once per device.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
char* g_scratch_ptr[kMaxDevices] = {};

hipError_t resolve_scratch(int device, char** out) {
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = static_cast<char*>(ptr);
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }
inline int round16(int r) { return (r + 15) / 16 * 16; }
inline int64_t round32(int64_t n) { return (n + 31) / 32 * 32; }

// carve-out of the ctx workspace for one layer; everything a step can need at the same time
struct Plan {
    size_t off_S, off_Q, off_B, off_pack, off_T, off_TpackT, off_xtt, off_qr, off_part, off_Ybuf, off_ce_ms, off_ce_tl, off_upd, off_ext, off_xqpart, total;
    int rp, nsplit;
    int64_t m_pad;
    int n_part;
    size_t part_count;   // doubles in the loss-partials region
};

// base: where this layer's carve-out starts inside the workspace (several layers side by side in the batched calls)
// fused_sketch: the range sketch comes out of the forward GEMM, one partial sum per 128-token tile
Plan make_plan(const agzo_layer& L, bool need_ybuf, bool ce = false, bool shared = false, size_t base = 0, bool fused_sketch = false) {
    Plan p;
    const bool bf = (L.dtype == AGZO_BF16);
    p.rp = round16(L.r);
    p.m_pad = fused_sketch ? gemm_bf16_sketch_mpad(L.n_tokens) : round32(L.n_tokens);
    p.nsplit = !bf ? 1 : fused_sketch ? gemm_bf16_sketch_splits(L.n_tokens) : xtt_num_splits(L.n_tokens, L.d_in);
    const int n_gemm = bf ? gemm_bf16_num_workgroups(L.n_tokens, L.d_out, !ce && !shared && L.tiling != AGZO_TILING_LARGE) : epilogue_f32_num_workgroups(L.n_tokens, L.d_out);
    p.n_part = n_gemm;
    size_t o = align_up(base);
    auto take = [&](size_t bytes) { size_t at = o; o += align_up(bytes); return at; };
    p.off_S = take((size_t)L.d_in * L.r * 4);
    p.off_Q = take((size_t)L.d_in * L.r * 4);
    p.off_B = take((size_t)L.d_in * L.r * 4);
    p.off_pack = take(bf ? (size_t)3 * p.rp * L.d_in * 2 : 0);
    p.off_T = take((size_t)L.n_tokens * L.r * 4);
    p.off_TpackT = take(bf ? (size_t)3 * p.rp * p.m_pad * 2 : 0);
    p.off_xtt = take(bf ? (size_t)p.nsplit * L.d_in * p.rp * 4 : 0);
    p.off_qr = take(qr_workspace_bytes(L.d_in, L.r));
    {
        size_t part = (size_t)n_gemm * 3;                                          // MSE: one double per tile and phase
        const size_t ce_part = (size_t)2 * L.n_tokens + 6 * ((L.n_tokens + 255) / 256);   // CE: (sum, count) pairs
        if (ce && ce_part > part) part = ce_part;
        p.part_count = part;
        p.off_part = take(part * 8);
    }
    p.off_ce_ms = take((ce && bf) ? (size_t)3 * gemm_bf16_ce_chunks(L.d_out) * L.n_tokens * 8 : 0);
    p.off_ce_tl = take((ce && bf) ? (size_t)3 * L.n_tokens * 4 : 0);
    p.off_upd = take(update_workspace_bytes(L.dtype, L.d_out, L.d_in, L.r));
    p.off_ext = take(bf ? gemm_bf16_ext_bytes(L.n_tokens, L.d_out, L.r) : 0);
    p.off_xqpart = take(bf ? xq_part_bytes(L.n_tokens, L.d_in, p.rp) : 0);
    p.off_Ybuf = take(need_ybuf ? (size_t)L.n_tokens * L.d_out * 4 : 0);
    p.total = o;
    return p;
}

int reserve(agzo_ctx* ctx, size_t bytes) {
    if (bytes <= ctx->ws_bytes) return 0;
    HIPCHK(hipStreamSynchronize(ctx->stream));
    if (ctx->ws) HIPCHK(hipFree(ctx->ws));
    ctx->ws = nullptr;
    ctx->ws_bytes = 0;
    void* p = nullptr;
    hipError_t e = hipMalloc(&p, bytes);
    if (e != hipSuccess) return fail(ctx, AGZO_ENOMEM, "workspace of %zu bytes: %s", bytes, hipGetErrorString(e));
    ctx->ws = static_cast<char*>(p);
    ctx->ws_bytes = bytes;
    return 0;
}

int check_layer(agzo_ctx* ctx, const agzo_layer* L, bool need_w) {
    if (!ctx) return AGZO_EINVAL;
    if (!L) return fail(ctx, AGZO_EINVAL, "layer descriptor is NULL");
    if (L->n_tokens < 1 || L->d_in < 1 || (need_w && L->d_out < 1))
        return fail(ctx, AGZO_EINVAL, "empty layer: n_tokens=%lld d_in=%lld d_out=%lld", (long long)L->n_tokens,
                    (long long)L->d_in, (long long)L->d_out);
    if (L->n_tokens > (1LL << 24) || L->d_in > (1LL << 24) || L->d_out > (1LL << 24))
        return fail(ctx, AGZO_EINVAL, "dimension above 2^24");
    if (L->r < 1 || L->r > kMaxRank) return fail(ctx, AGZO_EINVAL, "r=%d outside 1..%d", L->r, kMaxRank);
    if (L->r > L->n_tokens || L->r > L->d_in) return fail(ctx, AGZO_EINVAL, "r=%d exceeds min(n_tokens, d_in)", L->r);
    if (L->dtype != AGZO_F32 && L->dtype != AGZO_BF16) return fail(ctx, AGZO_EINVAL, "dtype %d", L->dtype);
    if (L->tiling != AGZO_TILING_AUTO && L->tiling != AGZO_TILING_LARGE) return fail(ctx, AGZO_EINVAL, "tiling %d", L->tiling);
    if (L->ldx < L->d_in || (need_w && L->ldw < L->d_in)) return fail(ctx, AGZO_EINVAL, "leading dimension below d_in");
    if (L->dtype == AGZO_BF16) {
        if (L->d_in % 8 || L->ldx % 8 || (need_w && L->ldw % 8))
            return fail(ctx, AGZO_EINVAL, "bf16 layers need d_in, ldx, ldw multiples of 8");
    }
    return 0;
}

// bf16 operands travel as 16-byte vectors (direct global -> LDS loads included) and the kernels build 32-bit byte
// offsets of up to 512 rows from a tile's corner
int check_operands(agzo_ctx* ctx, const agzo_layer* L, const void* W, const void* X) {
    if (L->dtype != AGZO_BF16) return 0;
    if ((reinterpret_cast<uintptr_t>(X) & 15) || (reinterpret_cast<uintptr_t>(W) & 15))
        return fail(ctx, AGZO_EINVAL, "bf16 X and W must be 16-byte aligned");
    if (L->ldx >= (1LL << 22) || (W && L->ldw >= (1LL << 22)))
        return fail(ctx, AGZO_EINVAL, "bf16 layers need ldx and ldw below 2^22 elements");
    return 0;
}

int check_y(agzo_ctx* ctx, const agzo_layer* L, const void* Y) {
    if (!Y) return 0;
    if (L->ldy < L->d_out) return fail(ctx, AGZO_EINVAL, "ldy below d_out");
    if (L->y_dtype == AGZO_F32) return 0;
    if (L->y_dtype == AGZO_BF16 && L->dtype == AGZO_BF16) return 0;
    return fail(ctx, AGZO_EINVAL, "y_dtype %d not supported for layer dtype %d", L->y_dtype, L->dtype);
}

int check_loss(agzo_ctx* ctx, const agzo_layer* L, const agzo_loss_spec* loss, const double* loss_dev) {
    if (!loss || loss->kind == AGZO_LOSS_NONE) return 0;
    if (loss->kind != AGZO_LOSS_MSE && loss->kind != AGZO_LOSS_CE)
        return fail(ctx, AGZO_EINVAL, "loss kind %d not supported", loss->kind);
    if (!loss->target || !loss_dev) return fail(ctx, AGZO_EINVAL, "loss needs a target and an output scalar");
    if (loss->kind == AGZO_LOSS_CE) return 0;
    if (loss->ldt < L->d_out) return fail(ctx, AGZO_EINVAL, "ldt below d_out");
    if (loss->target_dtype != AGZO_F32 && loss->target_dtype != AGZO_BF16)
        return fail(ctx, AGZO_EINVAL, "target dtype %d", loss->target_dtype);
    return 0;
}

// ---- internal building blocks; all take a ready workspace plan --------------------------------
inline float* wsf(agzo_ctx* c, size_t off) { return reinterpret_cast<float*>(c->ws + off); }
inline bf16_t* wsh(agzo_ctx* c, size_t off) { return reinterpret_cast<bf16_t*>(c->ws + off); }

// ---- sketches.  On the bf16 path a sketch first exists as per-token-range partials in the workspace
// (`splits`); they are summed either by the QR that consumes them or, when the caller wants S itself,
// by reduce_splits.  On the fp32 path S is produced directly.

// Omega^T planes -> splits (bf16) / S (fp32):  S = X^T Omega  (Alg. 1: Y <- H Omega)
int sketch_range(agzo_ctx* ctx, const agzo_layer& L, const Plan& p, const void* X, uint64_t seed, float* S) {
    hipStream_t st = ctx->stream;
    if (L.dtype == AGZO_BF16) {
        {
            ProfScope ps(ctx, AGZO_PROF_FILL);
            HIPCHK(launch_fill_normal_packT(wsh(ctx, p.off_TpackT), L.n_tokens, p.m_pad, L.r, p.rp, seed, AGZO_TAG_OMEGA, st));
        }
        ProfScope ps(ctx, AGZO_PROF_XTT);
        HIPCHK(launch_xtt_bf16(static_cast<const bf16_t*>(X), L.ldx, L.n_tokens, L.d_in, wsh(ctx, p.off_TpackT),
                               p.m_pad, p.rp, wsf(ctx, p.off_xtt), p.nsplit, st));
    } else {
        float* om = wsf(ctx, p.off_T);
        HIPCHK(launch_fill_normal(om, L.n_tokens, L.r, seed, AGZO_TAG_OMEGA, st));
        HIPCHK(launch_gemm_f32(static_cast<const float*>(X), 1, L.ldx, om, L.r, 1, S, L.r, L.d_in, L.r, L.n_tokens, st));
    }
    return 0;
}

// S = X^T (X Q)  (Alg. 1: Y <- H (H^T Q)).  bf16: Q must already sit in the workspace as planes.
int sketch_power(agzo_ctx* ctx, const agzo_layer& L, const Plan& p, const void* X, const float* Q, float* S) {
    hipStream_t st = ctx->stream;
    if (L.dtype == AGZO_BF16) {
        {
            ProfScope ps(ctx, AGZO_PROF_XQ);
            HIPCHK(launch_xq_bf16(static_cast<const bf16_t*>(X), L.ldx, L.n_tokens, L.d_in, wsh(ctx, p.off_pack), L.r,
                                  p.rp, nullptr, wsh(ctx, p.off_TpackT), p.m_pad, wsf(ctx, p.off_xqpart), st));
        }
        ProfScope ps(ctx, AGZO_PROF_XTT);
        HIPCHK(launch_xtt_bf16(static_cast<const bf16_t*>(X), L.ldx, L.n_tokens, L.d_in, wsh(ctx, p.off_TpackT),
                               p.m_pad, p.rp, wsf(ctx, p.off_xtt), p.nsplit, st));
    } else {
        const float* Xf = static_cast<const float*>(X);
        float* T = wsf(ctx, p.off_T);
        HIPCHK(launch_gemm_f32(Xf, L.ldx, 1, Q, L.r, 1, T, L.r, L.n_tokens, L.r, L.d_in, st));
        HIPCHK(launch_gemm_f32(Xf, 1, L.ldx, T, L.r, 1, S, L.r, L.d_in, L.r, L.n_tokens, st));
    }
    return 0;
}

int reduce_to_S(agzo_ctx* ctx, const agzo_layer& L, const Plan& p, float* S) {
    if (L.dtype == AGZO_BF16)
        HIPCHK(launch_reduce_splits(wsf(ctx, p.off_xtt), p.nsplit, L.d_in, p.rp, L.r, S, ctx->stream));
    return 0;
}

// Q = qr(S) for an explicit S; planes (nullable) also receive Q as bf16 planes
int op_qr(agzo_ctx* ctx, size_t off_qr, const float* S, int64_t d, int r, int rp, float* Q, bf16_t* planes,
          bool refine = true) {
    ProfScope ps(ctx, AGZO_PROF_QR);
    HIPCHK(launch_qr(S, nullptr, 0, rp, nullptr, d, r, Q, planes, ctx->ws + off_qr, ctx->flag, refine, ctx->stream));
    return 0;
}

// Q = qr(sum of the pending splits); the summed sketch is left in the workspace S
int op_qr_from_splits(agzo_ctx* ctx, const agzo_layer& L, const Plan& p, float* Q, bf16_t* planes, bool refine) {
    ProfScope ps(ctx, AGZO_PROF_QR);
    HIPCHK(launch_qr(nullptr, wsf(ctx, p.off_xtt), p.nsplit, p.rp, wsf(ctx, p.off_S), L.d_in, L.r, Q, planes,
                     ctx->ws + p.off_qr, ctx->flag, refine, ctx->stream));
    return 0;
}

// P = X B  (N x r).  planes_ready: B already sits in the workspace as planes (left there by the last QR)
int op_project(agzo_ctx* ctx, const agzo_layer& L, const Plan& p, const void* X, const float* B, float* P,
               bool planes_ready) {
    hipStream_t st = ctx->stream;
    if (L.dtype == AGZO_BF16) {
        if (!planes_ready) HIPCHK(launch_pack_planes(B, L.d_in, L.r, p.rp, wsh(ctx, p.off_pack), st));
        ProfScope ps(ctx, AGZO_PROF_XQ);
        HIPCHK(launch_xq_bf16(static_cast<const bf16_t*>(X), L.ldx, L.n_tokens, L.d_in, wsh(ctx, p.off_pack), L.r, p.rp,
                              P, nullptr, p.m_pad, wsf(ctx, p.off_xqpart), st));
    } else {
        HIPCHK(launch_gemm_f32(static_cast<const float*>(X), L.ldx, 1, B, L.r, 1, P, L.r, L.n_tokens, L.r, L.d_in, st));
    }
    return 0;
}

// Y = X W^T (+ eps (P) G^T), loss
// shared = true: one pass over X and W evaluates the loss at W, W + eps Z, W - eps Z -> loss_dev[0..2]
int op_forward(agzo_ctx* ctx, const agzo_layer& L, const Plan& p, const void* W, const void* X, const float* P,
               float eps_signed, uint64_t seed, void* Y, const agzo_loss_spec* loss, double* loss_dev,
               bool shared = false, int part_slot = 0, bool defer_finish = false, bool fused_sketch = false) {
    hipStream_t st = ctx->stream;
    GemmLossArgs la;
    const bool has_loss = loss && loss->kind != AGZO_LOSS_NONE;
    la.kind = has_loss ? loss->kind : AGZO_LOSS_NONE;
    la.target_dtype = has_loss ? loss->target_dtype : AGZO_F32;
    la.target = has_loss ? loss->target : nullptr;
    la.ldt = has_loss ? loss->ldt : 0;
    const bool ce = has_loss && loss->kind == AGZO_LOSS_CE;
    // squared error: a step keeps the tile partials of its forwards side by side (slot = 0, 1, 2) and finishes them in
    // one launch.  Cross-entropy: every loss is finished by launches of its own right behind the forward, so all of
    // them use the region from its start: (sum, count) per token (fp32 storage) or per 256 tokens and phase (bf16).
    {
        const size_t at = ce ? 0 : (size_t)part_slot * p.n_part;
        const size_t nblk = (size_t)((L.n_tokens + 255) / 256);
        const size_t need = !has_loss ? 0 : ce ? (L.dtype == AGZO_BF16 ? 2 * nblk * (shared ? 3 : 1) : 2 * (size_t)L.n_tokens)
                                               : (size_t)p.n_part * (shared ? 3 : 1);
        if (at + need > p.part_count)
            return fail(ctx, AGZO_EHIP, "internal: loss scratch of %zu doubles at %zu exceeds its region of %zu", need, at,
                        p.part_count);
        la.partials = reinterpret_cast<double*>(ctx->ws + p.off_part) + at;
    }
    const int32_t* ids = ce ? static_cast<const int32_t*>(loss->target) : nullptr;
    if (ce && L.dtype == AGZO_BF16) {
        la.ce_ms = ctx->ws + p.off_ce_ms;
        la.ce_tl = wsf(ctx, p.off_ce_tl);
    }
    if (L.dtype == AGZO_BF16) {
        GemmBf16Args a;
        a.X = static_cast<const bf16_t*>(X); a.ldx = L.ldx;
        a.W = static_cast<const bf16_t*>(W); a.ldw = L.ldw;
        a.M = L.n_tokens; a.N = L.d_out; a.K = L.d_in;
        a.Y = Y; a.y_dtype = L.y_dtype; a.ldy = L.ldy;
        a.P = P; a.r = L.r; a.eps_signed = eps_signed; a.seed = seed;
        a.loss = la;
        a.shared = shared;
        a.large_tiles = (L.tiling == AGZO_TILING_LARGE);
        a.ext_ws = P ? ctx->ws + p.off_ext : nullptr;
        if (fused_sketch) { a.sk_T = wsh(ctx, p.off_TpackT); a.sk_mpad = p.m_pad; a.sk_partial = wsf(ctx, p.off_xtt); }
        if (((ctx->prof >> AGZO_PROF_GEMM) & 1u) && ctx->clk_used < kClkSlots) a.clk = ctx->clk + 4 * ctx->clk_used++;
        {
            ProfScope ps(ctx, AGZO_PROF_GEMM);
            HIPCHK(launch_gemm_bf16(a, st));
        }
        if (ce)
            HIPCHK(launch_ce_combine(la.ce_ms, la.ce_tl, ids, L.n_tokens, L.d_out, gemm_bf16_ce_chunks(L.d_out), shared ? 3 : 1,
                                     la.partials, loss_dev, st));
    } else {
        float* Yf = Y ? static_cast<float*>(Y) : wsf(ctx, p.off_Ybuf);
        const int64_t ldy = Y ? L.ldy : L.d_out;
        HIPCHK(launch_gemm_f32(static_cast<const float*>(X), L.ldx, 1, static_cast<const float*>(W), 1, L.ldw, Yf, ldy,
                               L.n_tokens, L.d_out, L.d_in, st));
        if (shared) {
            // Y0 -> f0; Y0 + eps D -> f+; then - 2 eps D -> f-   (all in the stored fp32 Y buffer)
            GemmLossArgs l1 = la, l2 = la;
            l1.partials = la.partials + p.n_part;
            l2.partials = la.partials + 2 * p.n_part;
            HIPCHK(launch_epilogue_f32(Yf, ldy, L.n_tokens, L.d_out, nullptr, L.r, 0.f, seed, la, st));
            if (ce) HIPCHK(launch_ce_rows_f32(Yf, ldy, L.n_tokens, L.d_out, ids, la.partials, loss_dev + 0, st));
            HIPCHK(launch_epilogue_f32(Yf, ldy, L.n_tokens, L.d_out, P, L.r, eps_signed, seed, l1, st));
            if (ce) HIPCHK(launch_ce_rows_f32(Yf, ldy, L.n_tokens, L.d_out, ids, la.partials, loss_dev + 1, st));
            HIPCHK(launch_epilogue_f32(Yf, ldy, L.n_tokens, L.d_out, P, L.r, -2.f * eps_signed, seed, l2, st));
            if (ce) HIPCHK(launch_ce_rows_f32(Yf, ldy, L.n_tokens, L.d_out, ids, la.partials, loss_dev + 2, st));
        } else {
            HIPCHK(launch_epilogue_f32(Yf, ldy, L.n_tokens, L.d_out, P, L.r, eps_signed, seed, la, st));
            if (ce) HIPCHK(launch_ce_rows_f32(Yf, ldy, L.n_tokens, L.d_out, ids, la.partials, loss_dev, st));
        }
    }
    if (has_loss && !ce && !defer_finish)
        HIPCHK(launch_finish_loss(la.partials, p.n_part, 1.0 / ((double)L.n_tokens * (double)L.d_out), loss_dev,
                                  shared ? 3 : 1, st));
    return 0;
}

int check_update(agzo_ctx* ctx, const void* W, const float* B, int dtype, int64_t d_out, int64_t d_in, int64_t ldw, int r) {
    if (!W || !B) return fail(ctx, AGZO_EINVAL, "W or B is NULL");
    if (d_in < 1 || d_out < 1 || r < 1 || r > kMaxRank || r > d_in || ldw < d_in)
        return fail(ctx, AGZO_EINVAL, "bad layer shape");
    if (dtype != AGZO_F32 && dtype != AGZO_BF16) return fail(ctx, AGZO_EINVAL, "dtype %d", dtype);
    if (dtype == AGZO_BF16 && (d_in % 8 || ldw % 8 || (reinterpret_cast<uintptr_t>(W) & 15)))
        return fail(ctx, AGZO_EINVAL, "bf16 W needs d_in and ldw multiples of 8 and 16-byte aligned rows");
    if (dtype == AGZO_BF16 && ldw >= (1LL << 28)) return fail(ctx, AGZO_EINVAL, "bf16 W: ldw must be below 2^28");
    return 0;
}

int op_update(agzo_ctx* ctx, const agzo_layer& L, size_t off_upd, void* W, const float* B, uint64_t seed, float lr,
              const double* g_dev, float shift = 0.f) {
    ProfScope ps(ctx, AGZO_PROF_UPDATE);
    HIPCHK(launch_update(W, L.dtype, L.ldw, L.d_out, L.d_in, B, L.r, seed, lr, g_dev, ctx->ws + off_upd, ctx->stream, shift));
    return 0;
}

// Alg. 1.  On return (bf16) the workspace planes hold B.
int op_basis(agzo_ctx* ctx, const agzo_layer& L, const Plan& p, const void* X, int K, uint64_t seed, const float* S0,
             int flags, float* B) {
    const bool bf = (L.dtype == AGZO_BF16);
    float* S = wsf(ctx, p.off_S);
    float* Q = wsf(ctx, p.off_Q);
    bf16_t* planes = bf ? wsh(ctx, p.off_pack) : nullptr;
    const float* given = S0;      // an explicit first sketch, if any
    if (flags & AGZO_INIT_FEATURE) {
        HIPCHK(launch_fill_normal(Q, L.d_in, L.r, seed, AGZO_TAG_Q0, ctx->stream));
        if (bf) HIPCHK(launch_pack_planes(Q, L.d_in, L.r, p.rp, planes, ctx->stream));
        TRY(sketch_power(ctx, L, p, X, Q, S));
        given = nullptr;
    } else if (!given) {
        TRY(sketch_range(ctx, L, p, X, seed, S));
    }
    for (int k = 0; k <= K; ++k) {
        float* out = (k == K) ? B : Q;
        // iterates that are sketched again need a well-conditioned basis of the same span, not full orthonormality:
        // one Cholesky pass (same final QR factor, see qr.hip); the returned basis gets both passes
        const bool refine = (k == K);
        if (given) {
            TRY(op_qr(ctx, p.off_qr, given, L.d_in, L.r, p.rp, out, planes, refine));
            given = nullptr;
        } else if (bf) {
            TRY(op_qr_from_splits(ctx, L, p, out, planes, refine));
        } else {
            TRY(op_qr(ctx, p.off_qr, S, L.d_in, L.r, p.rp, out, nullptr, refine));
        }
        if (k < K) TRY(sketch_power(ctx, L, p, X, Q, S));
    }
    return 0;
}

// ---- several layers at once (Alg. 2: the base forward computes every layer's basis before the perturbed passes; the
// extractions are independent, so every stage of Alg. 1 is one launch for all layers) ----
struct LayerJob {
    agzo_layer L;
    Plan p;
    const void* X;
    uint64_t seed;
    const float* S0;
    float* B;          // where the basis goes
};

// one stage for the bf16 jobs idx[0..n): Omega^T planes + range sketch, or T = X Q planes + power sketch
int stage_sketch_many(agzo_ctx* ctx, const std::vector<LayerJob>& jobs, const int* idx, int n, bool range) {
    hipStream_t st = ctx->stream;
    if (range) {
        FillPackTArgs f[kBatchMax];
        for (int i = 0; i < n; ++i) {
            const LayerJob& j = jobs[idx[i]];
            f[i] = FillPackTArgs{wsh(ctx, j.p.off_TpackT), j.L.n_tokens, j.p.m_pad, j.L.r, j.p.rp, j.seed, AGZO_TAG_OMEGA};
        }
        ProfScope ps(ctx, AGZO_PROF_FILL);
        HIPCHK(launch_fill_normal_packT_many(f, n, st));
    } else {
        XqArgs q[kBatchMax];
        for (int i = 0; i < n; ++i) {
            const LayerJob& j = jobs[idx[i]];
            q[i] = XqArgs{static_cast<const bf16_t*>(j.X), j.L.ldx, j.L.n_tokens, j.L.d_in, wsh(ctx, j.p.off_pack), j.L.r, j.p.rp,
                          nullptr, wsh(ctx, j.p.off_TpackT), j.p.m_pad, wsf(ctx, j.p.off_xqpart)};
        }
        ProfScope ps(ctx, AGZO_PROF_XQ);
        HIPCHK(launch_xq_bf16_many(q, n, st));
    }
    XttArgs t[kBatchMax];
    for (int i = 0; i < n; ++i) {
        const LayerJob& j = jobs[idx[i]];
        t[i] = XttArgs{static_cast<const bf16_t*>(j.X), j.L.ldx, j.L.n_tokens, j.L.d_in, wsh(ctx, j.p.off_TpackT), j.p.m_pad, j.p.rp,
                       wsf(ctx, j.p.off_xtt), j.p.nsplit};
    }
    ProfScope ps(ctx, AGZO_PROF_XTT);
    HIPCHK(launch_xtt_bf16_many(t, n, st));
    return 0;
}

// Alg. 1 for every job.  bf16 jobs that share a padded rank go through the batched kernels, at most kBatchMax per
// launch; the others one by one.  On return every bf16 job's workspace planes hold its basis.
int basis_many_impl(agzo_ctx* ctx, const std::vector<LayerJob>& jobs, int K, int flags) {
    std::vector<char> done(jobs.size(), 0);
    for (size_t a = 0; a < jobs.size(); ++a) {
        if (done[a]) continue;
        const LayerJob& ja = jobs[a];
        if (ja.L.dtype != AGZO_BF16) {
            TRY(op_basis(ctx, ja.L, ja.p, ja.X, K, ja.seed, ja.S0, flags, ja.B));
            done[a] = 1;
            continue;
        }
        int idx[kBatchMax], n = 0;
        // (single columns are normalised rather than factored: launches of their own)
        for (size_t b = a; b < jobs.size() && n < kBatchMax; ++b)
            if (!done[b] && jobs[b].L.dtype == AGZO_BF16 && jobs[b].p.rp == ja.p.rp && (jobs[b].L.r == 1) == (ja.L.r == 1)) {
                idx[n++] = (int)b;
                done[b] = 1;
            }
        // first sketch: the feature-space start (Q0 from the seed, then a power sketch), a given S0, or the range sketch
        bool given[kBatchMax];
        int need_idx[kBatchMax], n_need = 0;
        for (int i = 0; i < n; ++i) {
            const LayerJob& j = jobs[idx[i]];
            given[i] = false;
            if (flags & AGZO_INIT_FEATURE) {
                HIPCHK(launch_fill_normal(wsf(ctx, j.p.off_Q), j.L.d_in, j.L.r, j.seed, AGZO_TAG_Q0, ctx->stream));
                HIPCHK(launch_pack_planes(wsf(ctx, j.p.off_Q), j.L.d_in, j.L.r, j.p.rp, wsh(ctx, j.p.off_pack), ctx->stream));
                need_idx[n_need++] = idx[i];
            } else if (j.S0) {
                given[i] = true;
            } else {
                need_idx[n_need++] = idx[i];
            }
        }
        if (n_need) TRY(stage_sketch_many(ctx, jobs, need_idx, n_need, !(flags & AGZO_INIT_FEATURE)));
        for (int k = 0; k <= K; ++k) {
            QrArgs q[kBatchMax];
            for (int i = 0; i < n; ++i) {
                const LayerJob& j = jobs[idx[i]];
                float* out = (k == K) ? j.B : wsf(ctx, j.p.off_Q);
                if (k == 0 && given[i])
                    q[i] = QrArgs{j.S0, nullptr, 0, j.p.rp, nullptr, j.L.d_in, j.L.r, out, wsh(ctx, j.p.off_pack), ctx->ws + j.p.off_qr};
                else
                    q[i] = QrArgs{nullptr, wsf(ctx, j.p.off_xtt), j.p.nsplit, j.p.rp, wsf(ctx, j.p.off_S), j.L.d_in, j.L.r, out,
                                  wsh(ctx, j.p.off_pack), ctx->ws + j.p.off_qr};
            }
            {
                ProfScope ps(ctx, AGZO_PROF_QR);
                HIPCHK(launch_qr_many(q, n, ctx->flag, k == K, ctx->stream));
            }
            if (k < K) TRY(stage_sketch_many(ctx, jobs, idx, n, false));
        }
    }
    return 0;
}

// P = X B for every bf16 job whose planes hold its basis (one launch per kBatchMax jobs of a padded rank)
int project_many(agzo_ctx* ctx, const std::vector<LayerJob>& jobs) {
    std::vector<char> done(jobs.size(), 0);
    for (size_t a = 0; a < jobs.size(); ++a) {
        if (done[a]) continue;
        const LayerJob& ja = jobs[a];
        if (ja.L.dtype != AGZO_BF16) {
            TRY(op_project(ctx, ja.L, ja.p, ja.X, ja.B, wsf(ctx, ja.p.off_T), true));
            done[a] = 1;
            continue;
        }
        XqArgs q[kBatchMax];
        int n = 0;
        for (size_t b = a; b < jobs.size() && n < kBatchMax; ++b) {
            const LayerJob& j = jobs[b];
            if (done[b] || j.L.dtype != AGZO_BF16 || j.p.rp != ja.p.rp) continue;
            q[n++] = XqArgs{static_cast<const bf16_t*>(j.X), j.L.ldx, j.L.n_tokens, j.L.d_in, wsh(ctx, j.p.off_pack), j.L.r, j.p.rp,
                            wsf(ctx, j.p.off_T), nullptr, j.p.m_pad, wsf(ctx, j.p.off_xqpart)};
            done[b] = 1;
        }
        ProfScope ps(ctx, AGZO_PROF_XQ);
        HIPCHK(launch_xq_bf16_many(q, n, ctx->stream));
    }
    return 0;
}

// checked items, workspace reserved: the factor fragments of all matrices start at workspace offset `off`.
// fp32 matrices one by one (no workspace); bf16 matrices with r = 1 in rank-1 sweeps of up to kBatchMax per launch (no
// workspace); the other bf16 matrices by padded rank, update_many_max() to a pair of launches
int update_many_at(agzo_ctx* ctx, const agzo_update_item* items, int n, size_t off) {
    for (int nk = -1; nk <= (kMaxRank + 15) / 16; ++nk) {
        std::vector<UpdateDesc> group;
        size_t group_bytes = 0;
        const int cap = (nk == 0) ? kBatchMax : update_many_max();
        auto flush = [&]() -> int {
            if (group.empty()) return 0;
            ProfScope ps(ctx, AGZO_PROF_UPDATE);
            if (nk == 0) {
                HIPCHK(launch_update_rank1_many(group.data(), (int)group.size(), ctx->stream));
            } else {
                HIPCHK(launch_update_many(group.data(), (int)group.size(), nk, ctx->ws + off, ctx->stream));
                off += group_bytes;
            }
            group.clear();
            group_bytes = 0;
            return 0;
        };
        for (int m = 0; m < n; ++m) {
            const agzo_update_item& u = items[m];
            if (nk < 0) {
                if (u.dtype != AGZO_F32) continue;
                ProfScope ps(ctx, AGZO_PROF_UPDATE);
                HIPCHK(launch_update(u.W, u.dtype, u.ldw, u.d_out, u.d_in, u.B, u.r, u.seed, u.lr, u.g_dev, nullptr, ctx->stream));
                continue;
            }
            if (u.dtype != AGZO_BF16) continue;
            if (nk == 0 ? u.r != 1 : (u.r == 1 || (u.r + 15) / 16 != nk)) continue;
            group.push_back(UpdateDesc{u.W, u.B, u.g_dev, u.ldw, u.d_out, u.d_in, u.seed, u.lr, u.r});
            if (nk > 0) group_bytes += update_workspace_bytes(u.dtype, u.d_out, u.d_in, u.r);
            if ((int)group.size() == cap) TRY(flush());
        }
        TRY(flush());
    }
    return AGZO_OK;
}

}  // namespace

extern "C" {

int agzo_create(agzo_ctx** out, void* hip_stream) {
    if (!out) return AGZO_EINVAL;
    agzo_ctx* ctx = new (std::nothrow) agzo_ctx;
    if (!ctx) return AGZO_ENOMEM;
    ctx->stream = static_cast<hipStream_t>(hip_stream);
    ctx->err[0] = 0;
    ctx->ws = nullptr;
    ctx->ws_bytes = 0;
    ctx->flag = nullptr;
    ctx->prof = 0;
    ctx->clk = nullptr;
    ctx->clk_used = 0;
    ctx->device = -1;
    ctx->static_scratch = nullptr;
    hipError_t e = hipGetDevice(&ctx->device);
    if (e == hipSuccess) e = resolve_scratch(ctx->device, &ctx->static_scratch);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&ctx->flag), 256);
    if (e == hipSuccess) e = hipMemset(ctx->flag, 0, 256);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&ctx->clk), kClkBytes);
    if (e == hipSuccess) e = hipMemset(ctx->clk, 0, kClkBytes);
    if (e != hipSuccess) {
        if (ctx->flag) (void)hipFree(ctx->flag);
        if (ctx->clk) (void)hipFree(ctx->clk);
        delete ctx;
        return AGZO_EHIP;
    }
    *out = ctx;
    return AGZO_OK;
}

void agzo_destroy(agzo_ctx* ctx) {
    if (!ctx) return;
    (void)hipStreamSynchronize(ctx->stream);
    if (ctx->ws) (void)hipFree(ctx->ws);
    if (ctx->flag) (void)hipFree(ctx->flag);
    if (ctx->clk) (void)hipFree(ctx->clk);
    for (auto& pc : ctx->pc) {
        for (hipEvent_t e : pc.start) (void)hipEventDestroy(e);
        for (hipEvent_t e : pc.stop) (void)hipEventDestroy(e);
    }
    delete ctx;
}

const char* agzo_last_error(const agzo_ctx* ctx) { return ctx ? ctx->err : "null context"; }

int agzo_check(agzo_ctx* ctx) {
    if (!ctx) return AGZO_EINVAL;
    HIPCHK(hipStreamSynchronize(ctx->stream));
    int h = 0;
    HIPCHK(hipMemcpy(&h, ctx->flag, sizeof(int), hipMemcpyDeviceToHost));
    if (h) {
        HIPCHK(hipMemset(ctx->flag, 0, sizeof(int)));
        return fail(ctx, AGZO_ENUMERIC, "Cholesky pivot <= 0: the sketch is rank deficient");
    }
    return AGZO_OK;
}

int agzo_profile_enable(agzo_ctx* ctx, int32_t mask) {
    if (!ctx) return AGZO_EINVAL;
    HIPCHK(hipStreamSynchronize(ctx->stream));
    ctx->prof = (uint32_t)mask & ((1u << AGZO_PROF_KINDS) - 1u);
    for (auto& pc : ctx->pc) pc.used = 0;
    ctx->clk_used = 0;
    return AGZO_OK;
}

namespace {
// rate of the constant counter that wall_clock64() reads, in Hz
int wall_rate(agzo_ctx* ctx, double* hz) {
    int dev = 0, khz = 0;
    HIPCHK(hipGetDevice(&dev));
    HIPCHK(hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev));
    if (khz <= 0) return fail(ctx, AGZO_EHIP, "device reports no wall clock rate");
    *hz = 1e3 * khz;
    return 0;
}
}  // namespace

int agzo_profile_clock(agzo_ctx* ctx, int64_t* launches, double* mean_ghz) {
    if (!ctx) return AGZO_EINVAL;
    if (!launches || !mean_ghz) return fail(ctx, AGZO_EINVAL, "bad clock query");
    HIPCHK(hipStreamSynchronize(ctx->stream));
    double hz = 0.0;
    TRY(wall_rate(ctx, &hz));
    std::vector<unsigned long long> h(4 * ctx->clk_used);
    if (ctx->clk_used) HIPCHK(hipMemcpy(h.data(), ctx->clk, h.size() * 8, hipMemcpyDeviceToHost));
    double cycles = 0.0, ticks = 0.0;
    for (size_t i = 0; i < ctx->clk_used; ++i) {
        cycles += (double)(h[4 * i + 2] - h[4 * i]);
        ticks += (double)(h[4 * i + 3] - h[4 * i + 1]);
    }
    *launches = (int64_t)ctx->clk_used;
    *mean_ghz = (ticks > 0.0) ? cycles / ticks * hz * 1e-9 : 0.0;
    return AGZO_OK;
}

int agzo_probe_mfma(agzo_ctx* ctx, const void* operands, int32_t duty, int32_t iters, double* tflops, double* clock_ghz) {
    if (!ctx) return AGZO_EINVAL;
    if (!operands || !tflops || !clock_ghz) return fail(ctx, AGZO_EINVAL, "NULL argument");
    if (duty < 1 || duty > 9 || iters < 1 || iters > (1 << 20)) return fail(ctx, AGZO_EINVAL, "need 1 <= duty <= 9 and 1 <= iters <= 2^20");
    double hz = 0.0;
    TRY(wall_rate(ctx, &hz));
    int dev = 0, cus = 0;
    HIPCHK(hipGetDevice(&dev));
    HIPCHK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    unsigned long long* rec = ctx->clk + 4 * kClkSlots;
    HIPCHK(launch_probe_mfma(operands, duty, iters, rec, ctx->stream));
    HIPCHK(hipStreamSynchronize(ctx->stream));
    unsigned long long h[4];
    HIPCHK(hipMemcpy(h, rec, sizeof(h), hipMemcpyDeviceToHost));
    const double seconds = (double)(h[3] - h[1]) / hz;
    if (seconds <= 0.0) return fail(ctx, AGZO_EHIP, "probe returned no time");
    // 16 MFMAs of 32x32x16 per issued group, 4 waves per workgroup, one workgroup per CU
    // (duty 9: the flop count of 8 groups from 256 instructions of 16x16x32)
    const double flops = 2.0 * 32 * 32 * 16 * 16.0 * (duty == 9 ? 8 : duty) * (double)iters * 4.0 * cus;
    *tflops = flops / seconds * 1e-12;
    *clock_ghz = (double)(h[2] - h[0]) / seconds * 1e-9;
    return AGZO_OK;
}

int agzo_profile_read(agzo_ctx* ctx, int32_t kind, int64_t* launches, double* total_ms) {
    if (!ctx) return AGZO_EINVAL;
    if (kind < 0 || kind >= AGZO_PROF_KINDS || !launches || !total_ms) return fail(ctx, AGZO_EINVAL, "bad profile query");
    HIPCHK(hipStreamSynchronize(ctx->stream));
    ProfClass& pc = ctx->pc[kind];
    double sum = 0.0;
    for (size_t i = 0; i < pc.used; ++i) {
        float ms = 0.f;
        HIPCHK(hipEventElapsedTime(&ms, pc.start[i], pc.stop[i]));
        sum += ms;
    }
    *launches = (int64_t)pc.used;
    *total_ms = sum;
    return AGZO_OK;
}

int agzo_philox_words(agzo_ctx* ctx, uint32_t* dst, int64_t rows, int32_t cols, uint64_t seed, uint32_t tag) {
    if (!ctx) return AGZO_EINVAL;
    if (rows < 0 || cols < 0 || rows > 0xFFFFFFFFLL) return fail(ctx, AGZO_EINVAL, "bad shape");
    if (!dst && rows * cols > 0) return fail(ctx, AGZO_EINVAL, "dst is NULL");
    HIPCHK(launch_philox_words(dst, rows, cols, seed, tag, ctx->stream));
    return AGZO_OK;
}

int agzo_fill_normal(agzo_ctx* ctx, float* dst, int64_t rows, int32_t cols, uint64_t seed, uint32_t tag) {
    if (!ctx) return AGZO_EINVAL;
    if (rows < 0 || cols < 0 || rows > 0xFFFFFFFFLL) return fail(ctx, AGZO_EINVAL, "bad shape");
    if (!dst && rows * cols > 0) return fail(ctx, AGZO_EINVAL, "dst is NULL");
    ProfScope ps(ctx, AGZO_PROF_FILL);
    HIPCHK(launch_fill_normal(dst, rows, cols, seed, tag, ctx->stream));
    return AGZO_OK;
}

int agzo_layer_forward_sketch(agzo_ctx* ctx, const agzo_layer* L, const void* W, const void* X, void* Y, int32_t mode,
                              const float* Q, uint64_t seed, float* S, const agzo_loss_spec* loss, double* loss_dev) {
    const bool gemm = (W != nullptr);
    TRY(check_layer(ctx, L, gemm));
    if (!X) return fail(ctx, AGZO_EINVAL, "X is NULL");
    TRY(check_operands(ctx, L, W, X));
    if (!gemm && (Y || (loss && loss->kind != AGZO_LOSS_NONE))) return fail(ctx, AGZO_EINVAL, "Y or loss without W");
    if (mode != AGZO_SKETCH_NONE && mode != AGZO_SKETCH_RANGE && mode != AGZO_SKETCH_POWER && mode != AGZO_SKETCH_RANGE_FUSED)
        return fail(ctx, AGZO_EINVAL, "sketch mode %d", mode);
    const bool fused = (mode == AGZO_SKETCH_RANGE_FUSED);
    if (fused) {
        const bool ce = loss && loss->kind == AGZO_LOSS_CE;
        if (!gemm || L->dtype != AGZO_BF16 || ce || !gemm_bf16_fuses_sketch(L->n_tokens, L->d_out, L->r, L->tiling == AGZO_TILING_LARGE))
            return fail(ctx, AGZO_EINVAL, "the fused range sketch needs a bf16 forward in the 128 x 128 tiling (few 256 x 256 tiles, "
                                          "no cross-entropy, tiling AUTO), r <= 16 and at most 8192 tokens");
    }
    if (mode != AGZO_SKETCH_NONE && !S) return fail(ctx, AGZO_EINVAL, "S is NULL");
    if (gemm) {
        TRY(check_y(ctx, L, Y));
        TRY(check_loss(ctx, L, loss, loss_dev));
    }
    const Plan p = make_plan(*L, gemm && L->dtype == AGZO_F32 && !Y, loss && loss->kind == AGZO_LOSS_CE, false, 0, fused);
    TRY(reserve(ctx, p.total));
    if (fused) {
        {
            ProfScope ps(ctx, AGZO_PROF_FILL);
            HIPCHK(launch_fill_normal_packT(wsh(ctx, p.off_TpackT), L->n_tokens, p.m_pad, L->r, p.rp, seed, AGZO_TAG_OMEGA, ctx->stream));
        }
        TRY(op_forward(ctx, *L, p, W, X, nullptr, 0.f, seed, Y, loss, loss_dev, false, 0, false, true));
        TRY(reduce_to_S(ctx, *L, p, S));
        return AGZO_OK;
    }
    if (gemm) TRY(op_forward(ctx, *L, p, W, X, nullptr, 0.f, seed, Y, loss, loss_dev));
    if (mode == AGZO_SKETCH_RANGE) {
        TRY(sketch_range(ctx, *L, p, X, seed, S));
        TRY(reduce_to_S(ctx, *L, p, S));
    }
    if (mode == AGZO_SKETCH_POWER) {
        if (!Q) {   // no Q given: the Gaussian feature-space start of the flagged variant, from the seed
            float* Q0 = wsf(ctx, p.off_Q);
            HIPCHK(launch_fill_normal(Q0, L->d_in, L->r, seed, AGZO_TAG_Q0, ctx->stream));
            Q = Q0;
        }
        if (L->dtype == AGZO_BF16)
            HIPCHK(launch_pack_planes(Q, L->d_in, L->r, p.rp, wsh(ctx, p.off_pack), ctx->stream));
        TRY(sketch_power(ctx, *L, p, X, Q, S));
        TRY(reduce_to_S(ctx, *L, p, S));
    }
    return AGZO_OK;
}

int agzo_qr(agzo_ctx* ctx, const float* S, int64_t d_in, int32_t r, float* Q) {
    if (!ctx) return AGZO_EINVAL;
    if (!S || !Q) return fail(ctx, AGZO_EINVAL, "S or Q is NULL");
    if (r < 1 || r > kMaxRank || d_in < r) return fail(ctx, AGZO_EINVAL, "need 1 <= r <= min(64, d_in)");
    TRY(reserve(ctx, qr_workspace_bytes(d_in, r)));
    return op_qr(ctx, 0, S, d_in, r, round16(r), Q, nullptr);
}

int agzo_basis(agzo_ctx* ctx, const agzo_layer* L, const void* X, int32_t K, uint64_t seed, const float* S0,
               int32_t flags, float* B) {
    TRY(check_layer(ctx, L, false));
    if (!X || !B) return fail(ctx, AGZO_EINVAL, "X or B is NULL");
    TRY(check_operands(ctx, L, nullptr, X));
    if (K < 0 || K > 64) return fail(ctx, AGZO_EINVAL, "K=%d outside 0..64", K);
    const Plan p = make_plan(*L, false);
    TRY(reserve(ctx, p.total));
    return op_basis(ctx, *L, p, X, K, seed, S0, flags, B);
}

int agzo_perturbed_forward(agzo_ctx* ctx, const agzo_layer* L, const void* W, const void* X, const float* B,
                           uint64_t seed, float eps_signed, void* Y, const agzo_loss_spec* loss, double* loss_dev) {
    TRY(check_layer(ctx, L, true));
    if (!W || !X || !B) return fail(ctx, AGZO_EINVAL, "W, X or B is NULL");
    TRY(check_operands(ctx, L, W, X));
    TRY(check_y(ctx, L, Y));
    TRY(check_loss(ctx, L, loss, loss_dev));
    const Plan p = make_plan(*L, L->dtype == AGZO_F32 && !Y, loss && loss->kind == AGZO_LOSS_CE);
    TRY(reserve(ctx, p.total));
    float* P = wsf(ctx, p.off_T);
    TRY(op_project(ctx, *L, p, X, B, P, false));
    return op_forward(ctx, *L, p, W, X, P, eps_signed, seed, Y, loss, loss_dev);
}

int agzo_update(agzo_ctx* ctx, const agzo_layer* L, void* W, const float* B, uint64_t seed, float lr,
                const double* g_dev) {
    if (!ctx) return AGZO_EINVAL;
    if (!L) return fail(ctx, AGZO_EINVAL, "layer descriptor is NULL");
    if (L->tiling != AGZO_TILING_AUTO && L->tiling != AGZO_TILING_LARGE) return fail(ctx, AGZO_EINVAL, "tiling %d", L->tiling);
    TRY(check_update(ctx, W, B, L->dtype, L->d_out, L->d_in, L->ldw, L->r));
    TRY(reserve(ctx, update_workspace_bytes(L->dtype, L->d_out, L->d_in, L->r)));
    TRY(op_update(ctx, *L, 0, W, B, seed, lr, g_dev));
    return AGZO_OK;
}

int agzo_update_noalloc(agzo_ctx* ctx, const agzo_layer* L, void* W, const float* B, uint64_t seed, float lr,
                        const double* g_dev) {
    if (!ctx) return AGZO_EINVAL;
    if (!L) return fail(ctx, AGZO_EINVAL, "layer descriptor is NULL");
    if (L->tiling != AGZO_TILING_AUTO && L->tiling != AGZO_TILING_LARGE) return fail(ctx, AGZO_EINVAL, "tiling %d", L->tiling);
    TRY(check_update(ctx, W, B, L->dtype, L->d_out, L->d_in, L->ldw, L->r));
    const size_t need = update_workspace_bytes(L->dtype, L->d_out, L->d_in, L->r);
    if (need > kStaticScratchBytes)
        return fail(ctx, AGZO_EINVAL, "factor fragments of this update take %zu bytes, the static scratch holds %zu",
                    need, kStaticScratchBytes);
    int dev = -1;
    HIPCHK(hipGetDevice(&dev));
    if (dev != ctx->device || !ctx->static_scratch)
        return fail(ctx, AGZO_EINVAL, "current device %d is not the context's device %d", dev, ctx->device);
    // the preparation launch rewrites every fragment the sweep reads, so nothing left by an earlier call is seen
    HIPCHK(launch_update(W, L->dtype, L->ldw, L->d_out, L->d_in, B, L->r, seed, lr, g_dev, ctx->static_scratch, ctx->stream));
    return AGZO_OK;
}

int agzo_update_many(agzo_ctx* ctx, const agzo_update_item* items, int32_t n) {
    if (!ctx) return AGZO_EINVAL;
    if (n < 0 || (n > 0 && !items)) return fail(ctx, AGZO_EINVAL, "bad item list");
    size_t need = 0;
    for (int m = 0; m < n; ++m) {
        const agzo_update_item& u = items[m];
        if (u.reserved != 0) return fail(ctx, AGZO_EINVAL, "item %d: reserved field must be 0", m);
        TRY(check_update(ctx, u.W, u.B, u.dtype, u.d_out, u.d_in, u.ldw, u.r));
        need += update_workspace_bytes(u.dtype, u.d_out, u.d_in, u.r);
    }
    TRY(reserve(ctx, need));
    return update_many_at(ctx, items, n, 0);
}

int agzo_dense_perturb(agzo_ctx* ctx, void* theta, int32_t dtype, int64_t rows, int64_t cols, int64_t ld, uint64_t seed,
                       float scale, const double* g_dev) {
    if (!ctx) return AGZO_EINVAL;
    if (rows < 0 || cols < 0 || ld < cols) return fail(ctx, AGZO_EINVAL, "bad shape %lld x %lld, ld %lld", (long long)rows, (long long)cols, (long long)ld);
    if (dtype != AGZO_F32 && dtype != AGZO_BF16) return fail(ctx, AGZO_EINVAL, "dtype %d", dtype);
    if (rows > 0xFFFFFFFFLL || (cols + 3) / 4 > 0xFFFFFFFFLL) return fail(ctx, AGZO_EINVAL, "rows and cols/4 must fit 32-bit counters");
    if (!theta && rows * cols > 0) return fail(ctx, AGZO_EINVAL, "theta is NULL");
    ProfScope ps(ctx, AGZO_PROF_FILL);
    HIPCHK(launch_dense_axpy(theta, dtype, rows, cols, ld, seed, scale, g_dev, ctx->stream));
    return AGZO_OK;
}

int agzo_two_point(agzo_ctx* ctx, double* out4_dev, float eps, int32_t flags) {
    if (!ctx) return AGZO_EINVAL;
    if (!out4_dev) return fail(ctx, AGZO_EINVAL, "out4_dev is NULL");
    if (!(eps > 0.f)) return fail(ctx, AGZO_EINVAL, "eps must be positive");
    HIPCHK(launch_two_point(out4_dev, eps, (flags & AGZO_ONE_SIDED) ? 1 : 0, ctx->stream));
    return AGZO_OK;
}

int agzo_basis_many(agzo_ctx* ctx, const agzo_basis_item* items, int32_t n, int32_t K, int32_t flags) {
    if (!ctx) return AGZO_EINVAL;
    if (n < 0 || (n > 0 && !items)) return fail(ctx, AGZO_EINVAL, "bad item list");
    if (K < 0 || K > 64) return fail(ctx, AGZO_EINVAL, "K=%d outside 0..64", K);
    std::vector<LayerJob> jobs((size_t)n);
    size_t total = 0;
    for (int m = 0; m < n; ++m) {
        const agzo_basis_item& it = items[m];
        TRY(check_layer(ctx, &it.layer, false));
        if (!it.X || !it.B) return fail(ctx, AGZO_EINVAL, "item %d: X or B is NULL", m);
        TRY(check_operands(ctx, &it.layer, nullptr, it.X));
        LayerJob& j = jobs[(size_t)m];
        j.L = it.layer; j.X = it.X; j.seed = it.seed; j.S0 = it.S0; j.B = it.B;
        j.p = make_plan(j.L, false, false, false, total);
        total = j.p.total;
    }
    TRY(reserve(ctx, total));
    return basis_many_impl(ctx, jobs, K, flags);
}

int agzo_step_many(agzo_ctx* ctx, const agzo_step_item* items, int32_t n, int32_t K, float eps, float lr, int32_t flags) {
    if (!ctx) return AGZO_EINVAL;
    if (n < 0 || (n > 0 && !items)) return fail(ctx, AGZO_EINVAL, "bad item list");
    if (K < 0 || K > 64) return fail(ctx, AGZO_EINVAL, "K=%d outside 0..64", K);
    if (!(eps > 0.f)) return fail(ctx, AGZO_EINVAL, "eps must be positive");
    if (flags & AGZO_NAIVE_INPLACE) return fail(ctx, AGZO_EINVAL, "the in-place comparator runs layer by layer (agzo_step)");
    const bool shared = (flags & AGZO_SHARED_FORWARD) != 0, one_sided = (flags & AGZO_ONE_SIDED) != 0;
    std::vector<LayerJob> jobs((size_t)n);
    size_t total = 0;
    for (int m = 0; m < n; ++m) {
        const agzo_step_item& it = items[m];
        TRY(check_layer(ctx, &it.layer, true));
        if (!it.W || !it.X || !it.out_dev) return fail(ctx, AGZO_EINVAL, "item %d: W, X or out_dev is NULL", m);
        if (it.loss.kind == AGZO_LOSS_NONE) return fail(ctx, AGZO_EINVAL, "item %d: a step needs a loss", m);
        TRY(check_loss(ctx, &it.layer, &it.loss, it.out_dev));
        TRY(check_operands(ctx, &it.layer, it.W, it.X));
        TRY(check_update(ctx, it.W, reinterpret_cast<const float*>(it.X) /* B is the call's own: any non-NULL */, it.layer.dtype, it.layer.d_out, it.layer.d_in, it.layer.ldw, it.layer.r));
        LayerJob& j = jobs[(size_t)m];
        j.L = it.layer; j.X = it.X; j.seed = it.seed; j.S0 = nullptr;
        j.p = make_plan(j.L, j.L.dtype == AGZO_F32, it.loss.kind == AGZO_LOSS_CE, shared, total);
        total = j.p.total;
    }
    size_t upd_bytes = 0;
    for (int m = 0; m < n; ++m)
        if (!items[m].B_out) upd_bytes += update_workspace_bytes(items[m].layer.dtype, items[m].layer.d_out, items[m].layer.d_in, items[m].layer.r);
    TRY(reserve(ctx, total + upd_bytes));
    for (int m = 0; m < n; ++m) jobs[(size_t)m].B = items[m].B_out ? items[m].B_out : wsf(ctx, jobs[(size_t)m].p.off_B);
    hipStream_t st = ctx->stream;
    auto forward = [&](int m, const float* P, float e, double* dst, bool sh, int slot) -> int {
        const agzo_step_item& it = items[m];
        const LayerJob& j = jobs[(size_t)m];
        return op_forward(ctx, j.L, j.p, it.W, it.X, P, e, it.seed, nullptr, &it.loss, dst, sh, slot, it.loss.kind == AGZO_LOSS_MSE);
    };
    // Alg. 2, part 1: the base forward of every layer, and every layer's basis from the same activations
    if (!shared)
        for (int m = 0; m < n; ++m) TRY(forward(m, nullptr, 0.f, items[m].out_dev, false, 0));
    TRY(basis_many_impl(ctx, jobs, K, flags & AGZO_INIT_FEATURE));
    // parts 2-3: the perturbed evaluations
    TRY(project_many(ctx, jobs));
    for (int m = 0; m < n; ++m) {
        const float* P = wsf(ctx, jobs[(size_t)m].p.off_T);
        if (shared) {
            TRY(forward(m, P, eps, items[m].out_dev, true, 0));
        } else {
            TRY(forward(m, P, +eps, items[m].out_dev + 1, false, 1));
            if (!one_sided) TRY(forward(m, P, -eps, items[m].out_dev + 2, false, 2));
        }
    }
    // the scalars, then every update in one batched call
    std::vector<agzo_update_item> upd;
    for (int m = 0; m < n; ++m) {
        const agzo_step_item& it = items[m];
        const LayerJob& j = jobs[(size_t)m];
        if (it.loss.kind == AGZO_LOSS_MSE)
            HIPCHK(launch_finish_two_point(reinterpret_cast<const double*>(ctx->ws + j.p.off_part), j.p.n_part,
                                           1.0 / ((double)j.L.n_tokens * (double)j.L.d_out), (shared || !one_sided) ? 3 : 2,
                                           it.out_dev, eps, one_sided ? 1 : 0, st));
        else
            HIPCHK(launch_two_point(it.out_dev, eps, one_sided ? 1 : 0, st));
        if (!it.B_out) {
            agzo_update_item u;
            u.W = it.W; u.B = j.B; u.g_dev = it.out_dev + 3;
            u.d_out = j.L.d_out; u.d_in = j.L.d_in; u.ldw = j.L.ldw; u.r = j.L.r; u.dtype = j.L.dtype;
            u.seed = it.seed; u.lr = lr; u.reserved = 0;
            upd.push_back(u);
        }
    }
    if (upd.empty()) return AGZO_OK;
    // the update's factor fragments go behind the layers' carve-outs, which still hold the bases
    size_t need = 0;
    for (const agzo_update_item& u : upd) need += update_workspace_bytes(u.dtype, u.d_out, u.d_in, u.r);
    if (total + need > ctx->ws_bytes) {
        // (reserve() would move the workspace and with it the bases: sized up front instead)
        return fail(ctx, AGZO_EHIP, "internal: update scratch was not reserved");
    }
    return update_many_at(ctx, upd.data(), (int)upd.size(), total);
}

namespace {
int check_glue(agzo_ctx* ctx, int64_t n, int64_t d, std::initializer_list<const void*> ptrs, std::initializer_list<int64_t> lds) {
    if (!ctx) return AGZO_EINVAL;
    if (n < 0 || d < 0 || d % 8) return fail(ctx, AGZO_EINVAL, "rows of %lld values: need a non-negative multiple of 8", (long long)d);
    for (const void* p : ptrs)
        if ((!p && n * d > 0) || (reinterpret_cast<uintptr_t>(p) & 15)) return fail(ctx, AGZO_EINVAL, "NULL or misaligned tensor");
    for (int64_t ld : lds)
        if (ld < d || ld % 8) return fail(ctx, AGZO_EINVAL, "leading dimension %lld below the row length or not a multiple of 8", (long long)ld);
    if (n > 0x7FFFFFFFLL) return fail(ctx, AGZO_EINVAL, "too many rows");
    return 0;
}
}  // namespace

int agzo_glue_rmsnorm(agzo_ctx* ctx, const void* x, int64_t ldx, void* y, int64_t ldy, const float* gain, int64_t n, int64_t d,
                      float eps) {
    TRY(check_glue(ctx, n, d, {x, y}, {ldx, ldy}));
    HIPCHK(launch_glue_rmsnorm(static_cast<const bf16_t*>(x), ldx, static_cast<bf16_t*>(y), ldy, gain, n, d, eps, ctx->stream));
    return AGZO_OK;
}

int agzo_glue_swiglu(agzo_ctx* ctx, const void* a, int64_t lda, const void* u, int64_t ldu, void* m, int64_t ldm, int64_t n,
                     int64_t d) {
    TRY(check_glue(ctx, n, d, {a, u, m}, {lda, ldu, ldm}));
    HIPCHK(launch_glue_swiglu(static_cast<const bf16_t*>(a), lda, static_cast<const bf16_t*>(u), ldu, static_cast<bf16_t*>(m), ldm,
                              n, d, ctx->stream));
    return AGZO_OK;
}

int agzo_glue_attention(agzo_ctx* ctx, const void* q, int64_t ldq, const void* k, int64_t ldk, const void* v, int64_t ldv,
                        void* out, int64_t ldo, int32_t n_seq, int32_t seq_len, int32_t n_heads, int32_t n_kv_heads,
                        float rope_theta) {
    if (!ctx) return AGZO_EINVAL;
    if (n_seq < 0 || seq_len < 0 || n_heads < 1 || n_kv_heads < 1 || n_heads % n_kv_heads || n_heads > 65535 || n_seq > 65535)
        return fail(ctx, AGZO_EINVAL, "bad attention shape: %d sequences of %d tokens, %d heads on %d kv heads", n_seq, seq_len, n_heads,
                    n_kv_heads);
    if (!(rope_theta > 1.f)) return fail(ctx, AGZO_EINVAL, "rope_theta must exceed 1");
    const int64_t n = (int64_t)n_seq * seq_len, dq = (int64_t)n_heads * 128, dkv = (int64_t)n_kv_heads * 128;
    TRY(check_glue(ctx, n, dq, {q, out}, {ldq, ldo}));
    TRY(check_glue(ctx, n, dkv, {k, v}, {ldk, ldv}));
    if (n == 0) return AGZO_OK;
    TRY(reserve(ctx, glue_attention_workspace_bytes(n_seq, seq_len, n_heads, n_kv_heads)));
    HIPCHK(launch_glue_attention(static_cast<const bf16_t*>(q), ldq, static_cast<const bf16_t*>(k), ldk, static_cast<const bf16_t*>(v), ldv,
                                 static_cast<bf16_t*>(out), ldo, n_seq, seq_len, n_heads, n_kv_heads, rope_theta, ctx->ws, ctx->stream));
    return AGZO_OK;
}

int agzo_glue_add(agzo_ctx* ctx, void* h, int64_t ldh, const void* delta, int64_t ldd, int64_t n, int64_t d) {
    TRY(check_glue(ctx, n, d, {h, delta}, {ldh, ldd}));
    HIPCHK(launch_glue_add(static_cast<bf16_t*>(h), ldh, static_cast<const bf16_t*>(delta), ldd, n, d, ctx->stream));
    return AGZO_OK;
}

// Alg. 2 for one layer.  B_out == NULL: the basis stays in the workspace and the update runs at the end;
// otherwise the basis goes to B_out and W is left as it was (the caller updates once g is final).
static int step_impl(agzo_ctx* ctx, const agzo_layer* L, void* W, const void* X, const agzo_loss_spec* loss, int32_t K,
                     float eps, float lr, uint64_t seed, int32_t flags, double* out_dev, float* B_out) {
    TRY(check_layer(ctx, L, true));
    if (!W || !X || !out_dev) return fail(ctx, AGZO_EINVAL, "W, X or out_dev is NULL");
    if (!loss || loss->kind == AGZO_LOSS_NONE) return fail(ctx, AGZO_EINVAL, "a step needs a loss");
    TRY(check_loss(ctx, L, loss, out_dev));
    if (K < 0 || K > 64) return fail(ctx, AGZO_EINVAL, "K=%d outside 0..64", K);
    if (!(eps > 0.f)) return fail(ctx, AGZO_EINVAL, "eps must be positive");
    TRY(check_operands(ctx, L, W, X));
    const Plan p = make_plan(*L, L->dtype == AGZO_F32, loss->kind == AGZO_LOSS_CE,
                             (flags & AGZO_SHARED_FORWARD) && !(flags & AGZO_NAIVE_INPLACE));
    TRY(reserve(ctx, p.total));
    hipStream_t st = ctx->stream;
    float* B = B_out ? B_out : wsf(ctx, p.off_B);
    const bool one_sided = (flags & AGZO_ONE_SIDED) != 0;
    // squared error: the forwards leave their tile partials side by side and one launch reduces them and forms g;
    // cross-entropy finishes each loss on its own and only g is left to do
    const bool mse = loss->kind == AGZO_LOSS_MSE;
    auto finish = [&](int nphase) -> int {
        if (mse)
            HIPCHK(launch_finish_two_point(reinterpret_cast<const double*>(ctx->ws + p.off_part), p.n_part,
                                           1.0 / ((double)L->n_tokens * (double)L->d_out), nphase, out_dev, eps,
                                           one_sided ? 1 : 0, st));
        else
            HIPCHK(launch_two_point(out_dev, eps, one_sided ? 1 : 0, st));
        return 0;
    };

    if ((flags & AGZO_SHARED_FORWARD) && !(flags & AGZO_NAIVE_INPLACE)) {
        // extraction first, then f0, f+ and f- from one pass over X and W (valid for a single layer:
        // all three evaluations read the same activations)
        TRY(op_basis(ctx, *L, p, X, K, seed, nullptr, flags & AGZO_INIT_FEATURE, B));
        float* P = wsf(ctx, p.off_T);
        TRY(op_project(ctx, *L, p, X, B, P, true));
        TRY(op_forward(ctx, *L, p, W, X, P, eps, seed, nullptr, loss, out_dev, true, 0, mse));
        TRY(finish(3));
        if (!B_out) TRY(op_update(ctx, *L, p.off_upd, W, B, seed, lr, out_dev + 3));
        return AGZO_OK;
    }
    // 1. base forward f0 and subspace extraction from the same activations (Alg. 2, part 1)
    TRY(op_forward(ctx, *L, p, W, X, nullptr, 0.f, seed, nullptr, loss, out_dev + 0, false, 0, mse));
    TRY(op_basis(ctx, *L, p, X, K, seed, nullptr, flags & AGZO_INIT_FEATURE, B));
    // 2. perturbed evaluations (Alg. 2, parts 2-3)
    if (flags & AGZO_NAIVE_INPLACE) {
        TRY(op_update(ctx, *L, p.off_upd, W, B, seed, -eps, nullptr));
        TRY(op_forward(ctx, *L, p, W, X, nullptr, 0.f, seed, nullptr, loss, out_dev + 1, false, 1, mse));
        if (!one_sided) {
            TRY(op_update(ctx, *L, p.off_upd, W, B, seed, 2.f * eps, nullptr));
            TRY(op_forward(ctx, *L, p, W, X, nullptr, 0.f, seed, nullptr, loss, out_dev + 2, false, 2, mse));
            TRY(op_update(ctx, *L, p.off_upd, W, B, seed, -eps, nullptr));
        } else if (B_out) {
            TRY(op_update(ctx, *L, p.off_upd, W, B, seed, eps, nullptr));
        } else {
            // Alg. 2 as printed: W still holds W + eps Z here, and the last line takes the perturbation out and applies
            // the update in one sweep, W <- W - (eps + lr g) Z
            TRY(finish(2));
            TRY(op_update(ctx, *L, p.off_upd, W, B, seed, lr, out_dev + 3, eps));
            return AGZO_OK;
        }
    } else {
        float* P = wsf(ctx, p.off_T);
        TRY(op_project(ctx, *L, p, X, B, P, true));
        TRY(op_forward(ctx, *L, p, W, X, P, +eps, seed, nullptr, loss, out_dev + 1, false, 1, mse));
        if (!one_sided) TRY(op_forward(ctx, *L, p, W, X, P, -eps, seed, nullptr, loss, out_dev + 2, false, 2, mse));
    }
    // 3. scalar g and the rank-r update
    TRY(finish(one_sided ? 2 : 3));
    if (!B_out) TRY(op_update(ctx, *L, p.off_upd, W, B, seed, lr, out_dev + 3));
    return AGZO_OK;
}

int agzo_step(agzo_ctx* ctx, const agzo_layer* L, void* W, const void* X, const agzo_loss_spec* loss, int32_t K,
              float eps, float lr, uint64_t seed, int32_t flags, double* out_dev) {
    return step_impl(ctx, L, W, X, loss, K, eps, lr, seed, flags, out_dev, nullptr);
}

int agzo_step_no_update(agzo_ctx* ctx, const agzo_layer* L, void* W, const void* X, const agzo_loss_spec* loss,
                        int32_t K, float eps, uint64_t seed, int32_t flags, double* out_dev, float* B_out) {
    if (ctx && !B_out) return fail(ctx, AGZO_EINVAL, "B_out is NULL");
    return step_impl(ctx, L, W, X, loss, K, eps, 0.f, seed, flags, out_dev, B_out);
}

}  // extern "C"
