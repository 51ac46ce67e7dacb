// In-place rank-r sweep of Alg. 2 (restore / update line, Eq. 10):
//     W[i][j] -= (lr * g + shift) * sum_k G[i][k] * B[j][k]
// (shift = 0 for the update alone; shift = eps makes it the printed last line of Alg. 2, which takes the perturbation
// out and applies the update in one sweep).
// W is read and written exactly once (HBM-bound); G is regenerated from the Philox seed (the d_out x d_in
// direction Z = G B^T never exists in memory); B (d_in x r fp32) is small and stays in L2.  fp32
// accumulation, one rounding to the storage type on the store.
#include "agzo_internal.h"

namespace agzo {

constexpr int UP_TI = 64;    // rows (d_out) per tile
constexpr int UP_TJ = 256;   // cols (d_in) per tile
constexpr int UP_TR = 8;     // rows per thread

// KC = number of k handled per register chunk; nchunk chunks cover r (zero padded)
template <int KC>
__global__ __launch_bounds__(256) void update_kernel(float* __restrict__ Wf, int64_t ldw, int64_t d_out, int64_t d_in,
                                                     const float* __restrict__ B, int r, int nchunk, uint32_t s_lo,
                                                     uint32_t s_hi, float lr, float shift,
                                                     const double* __restrict__ g_dev) {
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

    const float coef = -fmaf(lr, g_dev ? (float)(*g_dev) : 1.0f, shift);
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
        float* w = Wf + i * ldw + jc;
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

// ---------------------------------------------------------------------------
// bf16 storage: the outer product G B^T runs on the matrix cores (v_mfma_f32_32x32x16_bf16,
// K = r padded to 16).  A small preparation kernel writes both factors once, already split hi + lo in
// bf16 and already in the register order the matrix instruction wants (coef = -lr g folded into G), so
// the sweep itself holds no generator and no conversions of the factors: it is a read-add-write of W.
// Products hi*hi, hi*lo, lo*hi are accumulated: relative error 2^-16 of the increment.
//
// Roles: A-operand rows = rows i of W (G), B-operand columns = columns j of W (basis rows), interleaved
// over eight instructions (column c of instruction m is j = 8 c + m), so that a lane ends up with eight
// consecutive columns of one row (16 bytes) and a half-wave with 512 contiguous bytes.
// A wave owns 32 rows x 256 columns; the four waves of a workgroup share the basis fragments in LDS.
// ---------------------------------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
union FragU {
    uint4 u;
    bf16x8 v;
};

// eight fp32 values -> hi and lo bf16 fragments
__device__ __forceinline__ void split_frag(const float (&f)[8], FragU& hi, FragU& lo) {
    uint32_t h[4], l[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        h[i] = pack_bf16x2(f[2 * i], f[2 * i + 1]);
        const float r0 = f[2 * i] - __uint_as_float(h[i] << 16);
        const float r1 = f[2 * i + 1] - __uint_as_float(h[i] & 0xFFFF0000u);
        l[i] = pack_bf16x2(r0, r1);
    }
    hi.u = make_uint4(h[0], h[1], h[2], h[3]);
    lo.u = make_uint4(l[0], l[1], l[2], l[3]);
}

constexpr int UM_ROWS = 32;     // rows of W per wave
constexpr int UM_COLS = 256;    // columns of W per workgroup

// fragment stores (uint4 units):
//   Gf [row block ib][kc][plane][lane]        lane = (i % 32) + 32 * lh,      k = 16 kc + 8 lh + 0..7
//   Bf [col block jb][kc][plane][m][lane]     lane = c + 32 * lh, j = 256 jb + 8 c + m, same k
__device__ __forceinline__ void prep_fragment(uint4* __restrict__ Gf, uint4* __restrict__ Bf, int64_t n_g, int64_t n_b,
                                              int nk, int64_t d_out, int64_t d_in, const float* __restrict__ B, int r,
                                              uint32_t s_lo, uint32_t s_hi, float lr, float shift,
                                              const double* __restrict__ g_dev, int64_t t) {
    float f[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    FragU hi, lo;
    if (t < n_g) {
        const int lane = (int)(t & 63), kc = (int)((t >> 6) % nk);
        const int64_t ib = (t >> 6) / nk;
        const int64_t i = ib * UM_ROWS + (lane & 31);
        const int k0 = 16 * kc + 8 * (lane >> 5);
        if (i < d_out && k0 < r) {
            const float coef = -fmaf(lr, g_dev ? (float)(*g_dev) : 1.0f, shift);
            const float4 z0 = philox_normal4(s_lo, s_hi, AGZO_TAG_G, (uint32_t)i, (uint32_t)(k0 >> 2));
            f[0] = z0.x; f[1] = z0.y; f[2] = z0.z; f[3] = z0.w;
            if (k0 + 4 < r) {
                const float4 z1 = philox_normal4(s_lo, s_hi, AGZO_TAG_G, (uint32_t)i, (uint32_t)((k0 >> 2) + 1));
                f[4] = z1.x; f[5] = z1.y; f[6] = z1.z; f[7] = z1.w;
            }
#pragma unroll
            for (int q = 0; q < 8; ++q) f[q] = (k0 + q < r) ? coef * f[q] : 0.f;
        }
        split_frag(f, hi, lo);
        uint4* dst = Gf + ((ib * nk + kc) * 2) * 64 + lane;
        dst[0] = hi.u;
        dst[64] = lo.u;
    } else if (t < n_g + n_b) {
        const int64_t u = t - n_g;
        const int lane = (int)(u & 63), m = (int)((u >> 6) & 7), kc = (int)((u >> 9) % nk);
        const int64_t jb = (u >> 9) / nk;
        const int64_t j = jb * UM_COLS + 8 * (lane & 31) + m;
        const int k0 = 16 * kc + 8 * (lane >> 5);
        if (j < d_in) {
#pragma unroll
            for (int q = 0; q < 8; ++q)
                if (k0 + q < r) f[q] = B[j * r + k0 + q];
        }
        split_frag(f, hi, lo);
        uint4* dst = Bf + (((jb * nk + kc) * 2) * 8 + m) * 64 + lane;
        dst[0] = hi.u;
        dst[8 * 64] = lo.u;
    }
}

__global__ __launch_bounds__(256) void update_prep_kernel(uint4* __restrict__ Gf, uint4* __restrict__ Bf,
                                                          int64_t n_g, int64_t n_b, int nk, int64_t d_out,
                                                          int64_t d_in, const float* __restrict__ B, int r,
                                                          uint32_t s_lo, uint32_t s_hi, float lr, float shift,
                                                          const double* __restrict__ g_dev) {
    prep_fragment(Gf, Bf, n_g, n_b, nk, d_out, d_in, B, r, s_lo, s_hi, lr, shift, g_dev, (int64_t)blockIdx.x * 256 + threadIdx.x);
}

// Several matrices in one pair of launches (Alg. 2 updates every layer once the scalar g is known): the table is a
// kernel argument, a workgroup finds its matrix from the running block counts (uniform, a handful of scalar compares).
constexpr int UPD_MAX = 16;
struct UpdItem {
    bf16_t* W;
    uint4 *Gf, *Bf;
    const float* B;
    const double* g_dev;
    int64_t ldw, d_out, d_in, n_g, n_b;
    uint32_t prep_blk0, sweep_blk0;   // first workgroup of this matrix in the two launches
    uint32_t s_lo, s_hi;
    float lr;
    int r, njb, row_iters;
};
struct UpdBatch {
    int n;
    UpdItem it[UPD_MAX];
};

__global__ __launch_bounds__(256) void update_prep_many_kernel(const UpdBatch tb, int nk) {
    int m = 0;
    while (m + 1 < tb.n && blockIdx.x >= tb.it[m + 1].prep_blk0) ++m;
    const UpdItem& u = tb.it[m];
    prep_fragment(u.Gf, u.Bf, u.n_g, u.n_b, nk, u.d_out, u.d_in, u.B, u.r, u.s_lo, u.s_hi, u.lr, 0.f, u.g_dev,
                  (int64_t)(blockIdx.x - u.prep_blk0) * 256 + threadIdx.x);
}

template <int NK>   // NK = rp / 16
__device__ __forceinline__ void sweep_columns(bf16_t* __restrict__ W, int64_t ldw, int64_t d_out, int64_t d_in,
                                              const uint4* __restrict__ Gf, const uint4* __restrict__ Bf, int row_iters,
                                              int64_t jb, int64_t by) {
    extern __shared__ __align__(16) uint4 um_smem[];   // [NK][2][8][64]
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 31, lh = lane >> 5;
    {
        const uint4* src = Bf + jb * (NK * 2 * 8 * 64);
#pragma unroll
        for (int e = 0; e < NK * 4; ++e) um_smem[e * 256 + tid] = src[e * 256 + tid];
    }
    __syncthreads();
    const int64_t jc = jb * UM_COLS + 8 * c;     // this lane's eight consecutive columns
    const bool col_ok = jc < d_in;               // d_in is a multiple of 8: the piece is all in or all out
    const uint32_t voff = (uint32_t)((4 * lh * ldw + 8 * c) * 2);   // bytes from the tile's corner; ldw < 2^28 (host check)

    for (int it = 0; it < row_iters; ++it) {
        const int64_t ib = (by * row_iters + it) * 4 + wave;
        const int64_t i0 = ib * UM_ROWS;
        if (i0 >= d_out) break;                  // wave-uniform
        // this lane's rows: i0 + 8 (e / 4) + 4 lh + e % 4.  Addresses = a wave-uniform row base (scalar registers) plus
        // one 32-bit lane offset, instead of sixteen 64-bit pointers per lane
        char* tile;
        {   // kept in scalar registers: passing the halves through readfirstlane stops the compiler from turning the
            // sixteen row addresses into per-lane 64-bit induction variables of the row loop
            const uint64_t a = reinterpret_cast<uint64_t>(W + i0 * ldw + jb * UM_COLS);
            const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a), hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
            tile = reinterpret_cast<char*>(((uint64_t)hi << 32) | lo);
        }
        uint4 wv[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int64_t i = i0 + 8 * (e >> 2) + 4 * lh + (e & 3);
            wv[e] = make_uint4(0, 0, 0, 0);
            if (col_ok && i < d_out)
                wv[e] = *reinterpret_cast<const uint4*>(tile + (int64_t)(8 * (e >> 2) + (e & 3)) * ldw * 2 + voff);
        }
        floatx16 z[8];
#pragma unroll
        for (int m = 0; m < 8; ++m)
#pragma unroll
            for (int e = 0; e < 16; ++e) z[m][e] = 0.f;
#pragma unroll
        for (int kc = 0; kc < NK; ++kc) {
            FragU gh, gl;
            gh.u = Gf[((ib * NK + kc) * 2) * 64 + lane];
            gl.u = Gf[((ib * NK + kc) * 2 + 1) * 64 + lane];
#pragma unroll
            for (int m = 0; m < 8; ++m) {
                FragU bh, bl;
                bh.u = um_smem[((kc * 2) * 8 + m) * 64 + lane];
                bl.u = um_smem[((kc * 2 + 1) * 8 + m) * 64 + lane];
                z[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gh.v, bh.v, z[m], 0, 0, 0);
                z[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gh.v, bl.v, z[m], 0, 0, 0);
                z[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gl.v, bh.v, z[m], 0, 0, 0);
            }
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int64_t i = i0 + 8 * (e >> 2) + 4 * lh + (e & 3);
            if (!(col_ok && i < d_out)) continue;
            uint32_t* pw = reinterpret_cast<uint32_t*>(&wv[e]);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float w0 = __uint_as_float(pw[q] << 16), w1 = __uint_as_float(pw[q] & 0xFFFF0000u);
                pw[q] = pack_bf16x2(w0 + z[2 * q][e], w1 + z[2 * q + 1][e]);
            }
            *reinterpret_cast<uint4*>(tile + (int64_t)(8 * (e >> 2) + (e & 3)) * ldw * 2 + voff) = wv[e];
        }
    }
}

template <int NK>
__global__ __launch_bounds__(256, 2) void update_mfma_kernel(bf16_t* __restrict__ W, int64_t ldw, int64_t d_out,
                                                             int64_t d_in, const uint4* __restrict__ Gf,
                                                             const uint4* __restrict__ Bf, int row_iters) {
    sweep_columns<NK>(W, ldw, d_out, d_in, Gf, Bf, row_iters, blockIdx.x, blockIdx.y);
}

template <int NK>
__global__ __launch_bounds__(256, 2) void update_mfma_many_kernel(const UpdBatch tb) {
    int m = 0;
    while (m + 1 < tb.n && blockIdx.x >= tb.it[m + 1].sweep_blk0) ++m;
    const UpdItem& u = tb.it[m];
    const uint32_t local = blockIdx.x - u.sweep_blk0, by = local / (uint32_t)u.njb;
    sweep_columns<NK>(u.W, u.ldw, u.d_out, u.d_in, u.Gf, u.Bf, u.row_iters, local - by * (uint32_t)u.njb, by);
}

// ---------------------------------------------------------------------------
// bf16 storage, r = 1 (the paper's operating point): the perturbation is an outer product g b^T of two vectors, so the
// sweep is one read-multiply-add-write of W on the vector units with nothing prepared beforehand: a wave owns 16 rows
// x 512 columns, lane l < 16 regenerates the Gaussian value of row l once and the wave passes it around; a lane keeps
// its eight basis values in registers and has all 16 row pieces in flight before the first store.  Exact fp32
// products, one rounding to bf16.
// ---------------------------------------------------------------------------
constexpr int U1_ROWS = 16;     // rows per wave
constexpr int U1_COLS = 512;    // columns per wave (8 per lane)

__device__ __forceinline__ void update_rank1_bf16_body(bf16_t* __restrict__ W, int64_t ldw, int64_t d_out, int64_t d_in,
                                                       const float* __restrict__ B, uint32_t s_lo, uint32_t s_hi, float lr,
                                                       float shift, const double* __restrict__ g_dev, uint32_t bx, uint32_t by) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t i0 = ((int64_t)by * 4 + wave) * U1_ROWS;
    const int64_t jc = (int64_t)bx * U1_COLS + 8 * lane;
    if (i0 >= d_out) return;                               // wave-uniform
    const float coef = -fmaf(lr, g_dev ? (float)(*g_dev) : 1.0f, shift);
    float gmine = 0.f;
    if (lane < U1_ROWS && i0 + lane < d_out) gmine = coef * philox_normal4(s_lo, s_hi, AGZO_TAG_G, (uint32_t)(i0 + lane), 0u).x;
    const bool col_ok = jc < d_in;                          // d_in is a multiple of 8: the piece is all in or all out
    float b[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) b[c] = col_ok ? B[jc + c] : 0.f;
    uint4 wv[U1_ROWS];
#pragma unroll
    for (int e = 0; e < U1_ROWS; ++e) {
        wv[e] = make_uint4(0, 0, 0, 0);
        if (col_ok && i0 + e < d_out) wv[e] = *reinterpret_cast<const uint4*>(W + (i0 + e) * ldw + jc);
    }
#pragma unroll
    for (int e = 0; e < U1_ROWS; ++e) {
        const float g = __shfl(gmine, e);
        if (!(col_ok && i0 + e < d_out)) continue;
        uint32_t* pw = reinterpret_cast<uint32_t*>(&wv[e]);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float w0 = __uint_as_float(pw[q] << 16), w1 = __uint_as_float(pw[q] & 0xFFFF0000u);
            pw[q] = pack_bf16x2(w0 + g * b[2 * q], w1 + g * b[2 * q + 1]);
        }
        *reinterpret_cast<uint4*>(W + (i0 + e) * ldw + jc) = wv[e];
    }
}

__global__ __launch_bounds__(256) void update_rank1_bf16_kernel(bf16_t* __restrict__ W, int64_t ldw, int64_t d_out, int64_t d_in,
                                                                const float* __restrict__ B, uint32_t s_lo, uint32_t s_hi,
                                                                float lr, float shift, const double* __restrict__ g_dev) {
    update_rank1_bf16_body(W, ldw, d_out, d_in, B, s_lo, s_hi, lr, shift, g_dev, blockIdx.x, blockIdx.y);
}

struct U1Dev {
    bf16_t* W; int64_t ldw, d_out, d_in;
    const float* B; const double* g_dev;
    uint32_t s_lo, s_hi; float lr;
};
__global__ __launch_bounds__(256) void update_rank1_bf16_many_kernel(const KBatch<U1Dev> tb) {
    uint32_t bx, by;
    const U1Dev& a = tb.a[kbatch_find(tb, bx, by)];
    update_rank1_bf16_body(a.W, a.ldw, a.d_out, a.d_in, a.B, a.s_lo, a.s_hi, a.lr, 0.f, a.g_dev, bx, by);
}

size_t update_workspace_bytes(int dtype, int64_t d_out, int64_t d_in, int r) {
    if (dtype != AGZO_BF16) return 0;
    const int64_t nk = (r + 15) / 16;
    const int64_t nib = (d_out + UM_ROWS - 1) / UM_ROWS, njb = (d_in + UM_COLS - 1) / UM_COLS;
    return (size_t)(nib * nk * 2 * 64 + njb * nk * 2 * 8 * 64) * sizeof(uint4);
}

// more rows per workgroup (fewer reloads of the basis fragments) once the grid still covers the chip a few times
static int sweep_row_iters(int64_t njb, int64_t ngroups) {
    int row_iters = 1;
    while (row_iters < 4 && njb * (ngroups / (2 * row_iters)) >= 2048) row_iters *= 2;
    return row_iters;
}

template <int NK>
static hipError_t launch_mfma(bf16_t* W, int64_t ldw, int64_t d_out, int64_t d_in, const uint4* Gf, const uint4* Bf,
                              hipStream_t st) {
    const int64_t njb = (d_in + UM_COLS - 1) / UM_COLS;
    const int64_t ngroups = (d_out + 4 * UM_ROWS - 1) / (4 * UM_ROWS);
    const int row_iters = sweep_row_iters(njb, ngroups);
    dim3 grid((unsigned)njb, (unsigned)((ngroups + row_iters - 1) / row_iters));
    const size_t smem = (size_t)NK * 2 * 8 * 64 * sizeof(uint4);
    hipLaunchKernelGGL((update_mfma_kernel<NK>), grid, dim3(256), smem, st, W, ldw, d_out, d_in, Gf, Bf, row_iters);
    return hipGetLastError();
}

template <int KC>
static hipError_t launch_kc(float* W, int64_t ldw, int64_t d_out, int64_t d_in, const float* B, int r, int nchunk,
                            uint64_t seed, float lr, float shift, const double* g_dev, hipStream_t st) {
    dim3 grid((unsigned)((d_in + UP_TJ - 1) / UP_TJ), (unsigned)((d_out + UP_TI - 1) / UP_TI));
    const int rp = KC * nchunk;
    const size_t smem = (size_t)(UP_TI + UP_TJ) * rp * sizeof(float);
    static bool set = false;
    if (!set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(update_kernel<KC>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (UP_TI + UP_TJ) * kMaxRank * (int)sizeof(float));
        if (e != hipSuccess) return e;
        set = true;
    }
    hipLaunchKernelGGL((update_kernel<KC>), grid, dim3(256), smem, st, W, ldw, d_out, d_in, B, r, nchunk, (uint32_t)seed,
                       (uint32_t)(seed >> 32), lr, shift, g_dev);
    return hipGetLastError();
}

hipError_t launch_update(void* W, int dtype, int64_t ldw, int64_t d_out, int64_t d_in, const float* B, int r,
                         uint64_t seed, float lr, const double* g_dev, void* workspace, hipStream_t st, float shift) {
    if (d_out == 0 || d_in == 0) return hipSuccess;
    // fp32 storage keeps exact fp32 products (VALU); bf16 storage takes the matrix-core outer product
    if (dtype != AGZO_BF16) {
        float* Wf = static_cast<float*>(W);
        if (r <= 1) return launch_kc<1>(Wf, ldw, d_out, d_in, B, r, 1, seed, lr, shift, g_dev, st);
        if (r <= 2) return launch_kc<2>(Wf, ldw, d_out, d_in, B, r, 1, seed, lr, shift, g_dev, st);
        if (r <= 4) return launch_kc<4>(Wf, ldw, d_out, d_in, B, r, 1, seed, lr, shift, g_dev, st);
        if (r <= 8) return launch_kc<8>(Wf, ldw, d_out, d_in, B, r, 1, seed, lr, shift, g_dev, st);
        return launch_kc<16>(Wf, ldw, d_out, d_in, B, r, (r + 15) / 16, seed, lr, shift, g_dev, st);
    }
    if (r == 1) {
        const dim3 grid((unsigned)((d_in + U1_COLS - 1) / U1_COLS), (unsigned)((d_out + 4 * U1_ROWS - 1) / (4 * U1_ROWS)));
        hipLaunchKernelGGL(update_rank1_bf16_kernel, grid, dim3(256), 0, st, static_cast<bf16_t*>(W), ldw, d_out, d_in, B,
                           (uint32_t)seed, (uint32_t)(seed >> 32), lr, shift, g_dev);
        return hipGetLastError();
    }
    if (!workspace || ldw >= (1LL << 28)) return hipErrorInvalidValue;   // the sweep's lane offsets are 32-bit
    const int nk = (r + 15) / 16;
    const int64_t nib = (d_out + UM_ROWS - 1) / UM_ROWS, njb = (d_in + UM_COLS - 1) / UM_COLS;
    const int64_t n_g = nib * nk * 64, n_b = njb * nk * 8 * 64;
    uint4* Gf = static_cast<uint4*>(workspace);
    uint4* Bf = Gf + nib * nk * 2 * 64;
    hipLaunchKernelGGL(update_prep_kernel, dim3((unsigned)((n_g + n_b + 255) / 256)), dim3(256), 0, st, Gf, Bf, n_g, n_b,
                       nk, d_out, d_in, B, r, (uint32_t)seed, (uint32_t)(seed >> 32), lr, shift, g_dev);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    bf16_t* Wb = static_cast<bf16_t*>(W);
    switch (nk) {
        case 1: return launch_mfma<1>(Wb, ldw, d_out, d_in, Gf, Bf, st);
        case 2: return launch_mfma<2>(Wb, ldw, d_out, d_in, Gf, Bf, st);
        case 3: return launch_mfma<3>(Wb, ldw, d_out, d_in, Gf, Bf, st);
        default: return launch_mfma<4>(Wb, ldw, d_out, d_in, Gf, Bf, st);
    }
}

// bf16 matrices of one padded rank (nk = ceil(r / 16) the same for all), at most UPD_MAX of them: one preparation
// launch and one sweep for the lot.  The workspace holds the fragments of all of them back to back.
// bf16 matrices with r = 1, at most kBatchMax: one launch of the rank-1 sweep for all of them (no scratch)
hipError_t launch_update_rank1_many(const UpdateDesc* d, int n, hipStream_t st) {
    if (n < 0 || n > kBatchMax) return hipErrorInvalidValue;
    KBatch<U1Dev> tb;
    tb.n = 0;
    uint64_t blocks = 0;
    for (int m = 0; m < n; ++m) {
        if (d[m].d_out == 0 || d[m].d_in == 0) continue;
        if (d[m].r != 1) return hipErrorInvalidValue;
        const uint32_t gx = (uint32_t)((d[m].d_in + U1_COLS - 1) / U1_COLS);
        const uint64_t gy = (uint64_t)((d[m].d_out + 4 * U1_ROWS - 1) / (4 * U1_ROWS));
        tb.first[tb.n] = (uint32_t)blocks; tb.gx[tb.n] = gx;
        tb.a[tb.n++] = U1Dev{static_cast<bf16_t*>(d[m].W), d[m].ldw, d[m].d_out, d[m].d_in, d[m].B, d[m].g_dev,
                             (uint32_t)d[m].seed, (uint32_t)(d[m].seed >> 32), d[m].lr};
        blocks += gx * gy;
    }
    if (tb.n == 0) return hipSuccess;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(update_rank1_bf16_many_kernel, dim3((unsigned)blocks), dim3(256), 0, st, tb);
    return hipGetLastError();
}

hipError_t launch_update_many(const UpdateDesc* d, int n, int nk, void* workspace, hipStream_t st) {
    if (n < 1 || n > UPD_MAX || !workspace) return hipErrorInvalidValue;
    UpdBatch tb;
    tb.n = 0;
    uint4* ws = static_cast<uint4*>(workspace);
    int64_t prep_blocks = 0, sweep_blocks = 0;
    for (int m = 0; m < n; ++m) {
        if (d[m].d_out == 0 || d[m].d_in == 0) continue;
        if (d[m].ldw >= (1LL << 28)) return hipErrorInvalidValue;
        UpdItem& u = tb.it[tb.n++];
        const int64_t nib = (d[m].d_out + UM_ROWS - 1) / UM_ROWS, njb = (d[m].d_in + UM_COLS - 1) / UM_COLS;
        const int64_t ngroups = (d[m].d_out + 4 * UM_ROWS - 1) / (4 * UM_ROWS);
        u.W = static_cast<bf16_t*>(d[m].W);
        u.Gf = ws;
        u.Bf = ws + nib * nk * 2 * 64;
        ws = u.Bf + njb * nk * 2 * 8 * 64;
        u.B = d[m].B;
        u.g_dev = d[m].g_dev;
        u.ldw = d[m].ldw; u.d_out = d[m].d_out; u.d_in = d[m].d_in;
        u.n_g = nib * nk * 64; u.n_b = njb * nk * 8 * 64;
        u.s_lo = (uint32_t)d[m].seed; u.s_hi = (uint32_t)(d[m].seed >> 32);
        u.lr = d[m].lr; u.r = d[m].r;
        u.njb = (int)njb;
        u.row_iters = sweep_row_iters(njb, ngroups);
        u.prep_blk0 = (uint32_t)prep_blocks;
        u.sweep_blk0 = (uint32_t)sweep_blocks;
        prep_blocks += (u.n_g + u.n_b + 255) / 256;
        sweep_blocks += njb * ((ngroups + u.row_iters - 1) / u.row_iters);
    }
    if (tb.n == 0) return hipSuccess;
    if (prep_blocks > 0x7FFFFFFFLL || sweep_blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(update_prep_many_kernel, dim3((unsigned)prep_blocks), dim3(256), 0, st, tb, nk);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t smem = (size_t)nk * 2 * 8 * 64 * sizeof(uint4);
    const dim3 grid((unsigned)sweep_blocks);
    switch (nk) {
        case 1: hipLaunchKernelGGL((update_mfma_many_kernel<1>), grid, dim3(256), smem, st, tb); break;
        case 2: hipLaunchKernelGGL((update_mfma_many_kernel<2>), grid, dim3(256), smem, st, tb); break;
        case 3: hipLaunchKernelGGL((update_mfma_many_kernel<3>), grid, dim3(256), smem, st, tb); break;
        case 4: hipLaunchKernelGGL((update_mfma_many_kernel<4>), grid, dim3(256), smem, st, tb); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

int update_many_max() { return UPD_MAX; }

// Dense Gaussian sweep (Eq. 7, the branch for parameters that are not linear-layer weights; Alg. 2 perturb / restore /
// update lines): theta[i][j] += coef * z(i, j), z from Philox stream AGZO_TAG_DENSE, coef = scale * (*g_dev or 1).
// One thread = one Philox call = four consecutive columns of a row.  The generator (about 110 instructions per
// value) bounds this kernel, not the 4 - 8 bytes per value it moves.
template <typename T>
__global__ __launch_bounds__(256) void dense_axpy_kernel(T* __restrict__ theta, int64_t rows, int64_t cols, int64_t ld,
                                                         int64_t nquad, uint32_t s_lo, uint32_t s_hi, float scale,
                                                         const double* __restrict__ g_dev, int vec_ok) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= rows * nquad) return;
    const int64_t row = idx / nquad;
    const int64_t quad = idx - row * nquad;
    const float coef = g_dev ? (float)((double)scale * *g_dev) : scale;
    const float4 z4 = philox_normal4(s_lo, s_hi, AGZO_TAG_DENSE, (uint32_t)row, (uint32_t)quad);
    const float z[4] = {z4.x, z4.y, z4.z, z4.w};
    T* p = theta + row * ld + quad * 4;
    if (vec_ok) {
        if constexpr (sizeof(T) == 4) {
            float4 v = *reinterpret_cast<float4*>(p);
            v.x = fmaf(coef, z[0], v.x); v.y = fmaf(coef, z[1], v.y);
            v.z = fmaf(coef, z[2], v.z); v.w = fmaf(coef, z[3], v.w);
            *reinterpret_cast<float4*>(p) = v;
        } else {
            const uint2 w = *reinterpret_cast<uint2*>(p);
            const float a0 = fmaf(coef, z[0], __uint_as_float(w.x << 16)), a1 = fmaf(coef, z[1], __uint_as_float(w.x & 0xFFFF0000u));
            const float a2 = fmaf(coef, z[2], __uint_as_float(w.y << 16)), a3 = fmaf(coef, z[3], __uint_as_float(w.y & 0xFFFF0000u));
            *reinterpret_cast<uint2*>(p) = make_uint2(pack_bf16x2(a0, a1), pack_bf16x2(a2, a3));
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (quad * 4 + i >= cols) break;
            if constexpr (sizeof(T) == 4) p[i] = fmaf(coef, z[i], p[i]);
            else p[i] = f32_to_bf16(fmaf(coef, z[i], bf16_to_f32(p[i])));
        }
    }
}

hipError_t launch_dense_axpy(void* theta, int dtype, int64_t rows, int64_t cols, int64_t ld, uint64_t seed, float scale,
                             const double* g_dev, hipStream_t st) {
    if (rows == 0 || cols == 0) return hipSuccess;
    const int64_t nquad = (cols + 3) / 4;
    const int64_t items = rows * nquad;
    const dim3 grid((unsigned)((items + 255) / 256));
    const uintptr_t addr = reinterpret_cast<uintptr_t>(theta);
    if (dtype == AGZO_BF16) {
        const int vec = (cols % 4 == 0) && (ld % 4 == 0) && (addr % 8 == 0);
        hipLaunchKernelGGL(dense_axpy_kernel<bf16_t>, grid, dim3(256), 0, st, static_cast<bf16_t*>(theta), rows, cols, ld, nquad,
                           (uint32_t)seed, (uint32_t)(seed >> 32), scale, g_dev, vec);
    } else {
        const int vec = (cols % 4 == 0) && (ld % 4 == 0) && (addr % 16 == 0);
        hipLaunchKernelGGL(dense_axpy_kernel<float>, grid, dim3(256), 0, st, static_cast<float*>(theta), rows, cols, ld, nquad,
                           (uint32_t)seed, (uint32_t)(seed >> 32), scale, g_dev, vec);
    }
    return hipGetLastError();
}

}  // namespace agzo
