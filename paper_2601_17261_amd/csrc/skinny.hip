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
// xq: workgroup = 64 tokens, wave = 16 of them over the whole of d_in, so no cross-wave reduction.
// MFMA roles: A = X tile (rows = tokens, K = d_in), B = Q planes (K = d_in, cols = k); the three planes
// accumulate into the same registers.  X and the plane rows travel global -> LDS directly in 64-wide
// slices (one 128-byte line per row and slice, XOR-swizzled chunks) through a ring of XQ_STAGES slots,
// so that enough bytes are in flight per CU to cover the memory latency with four waves.
// ---------------------------------------------------------------------------
constexpr int XQ_TOK = 64;
constexpr int XQ_BK = 64;

__device__ __forceinline__ int xq_lds_off(int row, int c) { return row * 128 + ((c ^ ((row >> 1) & 7)) << 4); }

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}
// wait until at most n loads of this wave are outstanding (n is wave-uniform)
__device__ __forceinline__ void wait_vmcnt_dyn(int n) {
    switch (n) {
        case 0: wait_vmcnt<0>(); break;   case 3: wait_vmcnt<3>(); break;   case 4: wait_vmcnt<4>(); break;
        case 5: wait_vmcnt<5>(); break;   case 6: wait_vmcnt<6>(); break;   case 7: wait_vmcnt<7>(); break;
        case 8: wait_vmcnt<8>(); break;   case 9: wait_vmcnt<9>(); break;   case 10: wait_vmcnt<10>(); break;
        case 12: wait_vmcnt<12>(); break; case 14: wait_vmcnt<14>(); break; case 15: wait_vmcnt<15>(); break;
        case 16: wait_vmcnt<16>(); break; case 18: wait_vmcnt<18>(); break; case 20: wait_vmcnt<20>(); break;
        case 21: wait_vmcnt<21>(); break; case 24: wait_vmcnt<24>(); break; case 28: wait_vmcnt<28>(); break;
        default: wait_vmcnt<0>(); break;
    }
}

// bx: token block, by / ny: this workgroup's share of d_in (ny = 1: all of it)
// ring depth: DEEP = one workgroup per CU with as many slices in flight as LDS holds; otherwise a shallower ring that
// lets two workgroups share a CU, for launches with at least two workgroups per CU (several layers at once): while one
// waits at its barrier or on its fragment reads the other multiplies
template <int NB, bool DEEP>
struct XqRing { static constexpr int STAGES = DEEP ? ((NB == 1) ? 8 : (NB == 2) ? 6 : 4) : ((NB == 1) ? 5 : (NB == 2) ? 3 : 4); };

template <int NB, bool DEEP>
__device__ __forceinline__ void xq_bf16_body(const bf16_t* __restrict__ X, int64_t ldx, int64_t M, int64_t K,
                                             const bf16_t* __restrict__ Qpack, int r, float* __restrict__ T,
                                             bf16_t* __restrict__ TpackT, int64_t m_pad, float* __restrict__ part,
                                             uint32_t bx, uint32_t by, uint32_t ny) {
    constexpr int RP = NB * 16;
    constexpr int QROWS = 3 * RP;                          // plane rows: (plane, k)
    constexpr int NGROUP = XQ_TOK / 8 + QROWS / 8;         // 8-row groups per slice: X first, then the planes
    constexpr int SLOT = (XQ_TOK + QROWS) * 128;           // bytes per ring slot
    constexpr int STAGES = XqRing<NB, DEEP>::STAGES;
    extern __shared__ __align__(16) char xq_smem[];
    typedef __attribute__((address_space(3))) void* lptr_t;
    typedef const __attribute__((address_space(1))) void* gptr_t;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lm = lane & 15, lg = lane >> 4;
    const int64_t t0 = (int64_t)bx * XQ_TOK;

    floatx4 acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[nb] = floatx4{0.f, 0.f, 0.f, 0.f};

    // this wave's row groups g = wave, wave + 4, ...: per-lane source pointers (row of the group, swizzled chunk)
    constexpr int MAXG = (NGROUP + 3) / 4;
    const int ng = (NGROUP - wave + 3) / 4;                // groups of this wave
    const bf16_t* src[MAXG];
#pragma unroll
    for (int i = 0; i < MAXG; ++i) {
        const int g = min(wave + 4 * i, NGROUP - 1);
        const int row = 8 * g + (lane >> 3);
        const int c = (lane & 7) ^ ((row >> 1) & 7);
        if (row < XQ_TOK) src[i] = X + min(t0 + row, M - 1) * ldx + c * 8;
        else src[i] = Qpack + (int64_t)(row - XQ_TOK) * K + c * 8;
    }
    // few tokens: gridDim.y workgroups share a token block, each taking a contiguous run of d_in slices, and leave
    // partial sums in `part` for xq_finish_kernel (a single workgroup per block would walk d_in alone, bound by latency)
    const int nsplit = (int)ny, split = (int)by;
    const int nfull_all = (int)(K / XQ_BK);
    const int kbeg = (int)((int64_t)nfull_all * split / nsplit);
    const int nfull = (int)((int64_t)nfull_all * (split + 1) / nsplit) - kbeg;      // this workgroup's slices
    const bool tail = (K % XQ_BK) != 0 && split == nsplit - 1;
    auto issue = [&](int kt, int slot) __attribute__((always_inline)) {
        char* base = xq_smem + slot * SLOT + wave * 1024;
#pragma unroll
        for (int i = 0; i < MAXG; ++i)
            if (i < ng)
                __builtin_amdgcn_global_load_lds((gptr_t)(src[i] + (int64_t)(kbeg + kt) * XQ_BK), (lptr_t)(base + i * 4096), 16, 0, 0);
    };
    // Fragment reads go through inline assembly: for a plain LDS load the compiler, which cannot tell the ring's slots
    // apart, first waits for every direct load in flight (vmcnt(0)) and so collapses the ring to one slice.  The
    // waits that are needed are the explicit ones around the barrier and the lgkmcnt below.
    auto lds_read16 = [&](const char* ptr) __attribute__((always_inline)) {
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        u32x4 v;
        const uint32_t addr = (uint32_t)(uintptr_t)(lptr_t)ptr;
        asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr));
        return v;
    };
    auto multiply = [&](int slot, bool dma) __attribute__((always_inline)) {
        const char* xs = xq_smem + slot * SLOT;
        const char* qs = xs + XQ_TOK * 128;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
            u32x4 a, b[NB][3];
            a = lds_read16(xs + xq_lds_off(wave * 16 + lm, sub * 4 + lg));
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int pl = 0; pl < 3; ++pl) b[nb][pl] = lds_read16(qs + xq_lds_off(pl * RP + nb * 16 + lm, sub * 4 + lg));
            // the wait names every loaded register as an in/out operand, so nothing that uses them can move above it
            if constexpr (NB == 1)
                asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a), "+v"(b[0][0]), "+v"(b[0][1]), "+v"(b[0][2]) :: "memory");
            else if constexpr (NB == 2)
                asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a), "+v"(b[0][0]), "+v"(b[0][1]), "+v"(b[0][2]), "+v"(b[1][0]),
                             "+v"(b[1][1]), "+v"(b[1][2]) :: "memory");
            else if constexpr (NB == 3)
                asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a), "+v"(b[0][0]), "+v"(b[0][1]), "+v"(b[0][2]), "+v"(b[1][0]),
                             "+v"(b[1][1]), "+v"(b[1][2]), "+v"(b[2][0]), "+v"(b[2][1]), "+v"(b[2][2]) :: "memory");
            else
                asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a), "+v"(b[0][0]), "+v"(b[0][1]), "+v"(b[0][2]), "+v"(b[1][0]),
                             "+v"(b[1][1]), "+v"(b[1][2]), "+v"(b[2][0]), "+v"(b[2][1]), "+v"(b[2][2]), "+v"(b[3][0]),
                             "+v"(b[3][1]), "+v"(b[3][2]) :: "memory");
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int pl = 0; pl < 3; ++pl)
                    acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b[nb][pl]),
                                                                      acc[nb], 0, 0, 0);
        }
        (void)dma;
    };
    // ring: slices kt .. kt + STAGES - 2 in flight while slice kt is multiplied
#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s)
        if (s < nfull) issue(s, s);
    int slot = 0;
    for (int kt = 0; kt < nfull; ++kt) {
        // this wave's loads of slice kt have landed when at most (younger slices in flight) * ng are outstanding
        const int younger = min(STAGES - 2, nfull - 1 - kt);
        wait_vmcnt_dyn(younger * ng);
        // everybody's loads of slice kt have landed; the slot of slice kt-1 is free.  A bare barrier: __syncthreads()
        // would first wait for every load in flight and collapse the ring to one slice.
        __builtin_amdgcn_s_waitcnt(0xC07F);                // lgkmcnt(0)
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        if (kt + STAGES - 1 < nfull) issue(kt + STAGES - 1, (slot + STAGES - 1) % STAGES);
        multiply(slot, true);
        slot = (slot + 1 == STAGES) ? 0 : slot + 1;
    }
    if (tail) {
        // ragged end of d_in: the threads copy it themselves, zero past d_in
        __syncthreads();
        char* base = xq_smem;                              // slot 0 (all loads have landed and were consumed)
        for (int e = tid; e < (XQ_TOK + QROWS) * 8; e += 256) {
            const int row = e >> 3, c = e & 7;
            const int64_t kcol = (int64_t)nfull_all * XQ_BK + c * 8;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (kcol < K) {
                const bf16_t* p = (row < XQ_TOK) ? X + min(t0 + row, M - 1) * ldx + kcol
                                                 : Qpack + (int64_t)(row - XQ_TOK) * K + kcol;
                v = *reinterpret_cast<const uint4*>(p);
            }
            *reinterpret_cast<uint4*>(base + xq_lds_off(row, c)) = v;
        }
        __syncthreads();
        multiply(0, false);
    }
    // D layout: row (token) = 4*(lane/16) + e, col (k) = lane%16
    if (part != nullptr) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int64_t t = t0 + wave * 16 + lg * 4 + e;
                if (t < m_pad) part[((int64_t)split * m_pad + t) * RP + nb * 16 + lm] = acc[nb][e];
            }
        return;
    }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int k = nb * 16 + lm;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int64_t t = t0 + wave * 16 + lg * 4 + e;
            const float v = (t < M && k < r) ? acc[nb][e] : 0.f;
            if (t < M && k < r && T != nullptr) T[t * r + k] = v;
            if (TpackT != nullptr && t < m_pad) {
                bf16_t hi, mid, lo;
                split3_bf16(v, hi, mid, lo);
                TpackT[((int64_t)0 * RP + k) * m_pad + t] = hi;
                TpackT[((int64_t)1 * RP + k) * m_pad + t] = mid;
                TpackT[((int64_t)2 * RP + k) * m_pad + t] = lo;
            }
        }
    }
}

template <int NB>
__global__ __launch_bounds__(256) void xq_bf16_kernel(const bf16_t* __restrict__ X, int64_t ldx, int64_t M, int64_t K,
                                                      const bf16_t* __restrict__ Qpack, int r, float* __restrict__ T,
                                                      bf16_t* __restrict__ TpackT, int64_t m_pad, float* __restrict__ part) {
    xq_bf16_body<NB, true>(X, ldx, M, K, Qpack, r, T, TpackT, m_pad, part, blockIdx.x, blockIdx.y, gridDim.y);
}

// several products per launch (the layers of a model): what one launch of the kernel above needs, per product
struct XqDev {
    const bf16_t* X; int64_t ldx, M, K;
    const bf16_t* Qpack; int r;
    float* T; bf16_t* TpackT; int64_t m_pad; float* part;   // part: NULL unless ns > 1
    int ns; int64_t rows;
};
template <int NB, bool DEEP>
__global__ __launch_bounds__(256) void xq_bf16_many_kernel(const KBatch<XqDev> tb) {
    uint32_t bx, by;
    const XqDev& a = tb.a[kbatch_find(tb, bx, by)];
    xq_bf16_body<NB, DEEP>(a.X, a.ldx, a.M, a.K, a.Qpack, a.r, a.T, a.TpackT, a.m_pad, a.part, bx, by, (uint32_t)a.ns);
}

// sums the d_in splits of xq in fixed order and writes what the unsplit kernel's epilogue writes; one thread per (t, k)
__device__ __forceinline__ void xq_finish_body(const float* __restrict__ part, int nsplit, int64_t rows, int64_t M,
                                               int64_t m_pad, int r, int rp, float* __restrict__ T,
                                               bf16_t* __restrict__ TpackT, uint32_t bx) {
    const int64_t idx = (int64_t)bx * 256 + threadIdx.x;
    if (idx >= rows * rp) return;
    const int64_t t = idx / rp;
    const int k = (int)(idx - t * rp);
    float v = 0.f;
    if (t < M && k < r)
        for (int s = 0; s < nsplit; ++s) v += part[((int64_t)s * m_pad + t) * rp + k];
    if (t < M && k < r && T != nullptr) T[t * r + k] = v;
    if (TpackT != nullptr && t < m_pad) {
        bf16_t hi, mid, lo;
        split3_bf16(v, hi, mid, lo);
        TpackT[((int64_t)0 * rp + k) * m_pad + t] = hi;
        TpackT[((int64_t)1 * rp + k) * m_pad + t] = mid;
        TpackT[((int64_t)2 * rp + k) * m_pad + t] = lo;
    }
}

__global__ __launch_bounds__(256) void xq_finish_kernel(const float* __restrict__ part, int nsplit, int64_t rows, int64_t M,
                                                        int64_t m_pad, int r, int rp, float* __restrict__ T,
                                                        bf16_t* __restrict__ TpackT) {
    xq_finish_body(part, nsplit, rows, M, m_pad, r, rp, T, TpackT, blockIdx.x);
}

__global__ __launch_bounds__(256) void xq_finish_many_kernel(const KBatch<XqDev> tb, int rp) {
    uint32_t bx, by;
    const XqDev& a = tb.a[kbatch_find(tb, bx, by)];
    xq_finish_body(a.part, a.ns, a.rows, a.M, a.m_pad, a.r, rp, a.T, a.TpackT, bx);
}

// number of d_in splits for M tokens (1 = the token blocks alone fill the chip, or d_in is too short to share)
static int xq_splits(int64_t rows, int64_t K) {
    const int64_t blocks = (rows + XQ_TOK - 1) / XQ_TOK;
    const int64_t slices = K / XQ_BK;
    if (blocks >= 128 || slices < 16) return 1;
    int64_t want = 256 / blocks;
    if (want > slices / 8) want = slices / 8;      // at least eight slices each: the depth of the load ring
    if (want > 16) want = 16;
    return (int)(want < 1 ? 1 : want);
}

size_t xq_part_bytes(int64_t M, int64_t K, int rp) {
    const int64_t m_pad = (M + 31) / 32 * 32;
    const int ns = xq_splits(m_pad, K);
    return ns > 1 ? (size_t)ns * m_pad * rp * sizeof(float) : 0;
}

template <int NB>
static hipError_t launch_xq_nb(dim3 grid, hipStream_t st, const bf16_t* X, int64_t ldx, int64_t M, int64_t K,
                               const bf16_t* Qpack, int r, float* T, bf16_t* TpackT, int64_t m_pad, float* part) {
    constexpr int stages = (NB == 1) ? 8 : (NB == 2) ? 6 : 4;
    const int smem = stages * (XQ_TOK + 3 * NB * 16) * 128;
    static bool set = false;
    if (!set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(xq_bf16_kernel<NB>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        set = true;
    }
    hipLaunchKernelGGL(xq_bf16_kernel<NB>, grid, dim3(256), smem, st, X, ldx, M, K, Qpack, r, T, TpackT, m_pad, part);
    return hipGetLastError();
}

template <int NB, bool DEEP>
static hipError_t launch_xq_many_ring(const KBatch<XqDev>& tb, unsigned blocks, hipStream_t st) {
    const int smem = XqRing<NB, DEEP>::STAGES * (XQ_TOK + 3 * NB * 16) * 128;
    static bool set = false;
    if (!set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(xq_bf16_many_kernel<NB, DEEP>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        set = true;
    }
    hipLaunchKernelGGL((xq_bf16_many_kernel<NB, DEEP>), dim3(blocks), dim3(256), smem, st, tb);
    return hipGetLastError();
}
template <int NB>
static hipError_t launch_xq_many_nb(const KBatch<XqDev>& tb, unsigned blocks, hipStream_t st) {
    // (the result does not depend on the ring's depth: same slices, same order)
    if (NB <= 2 && blocks >= 512) return launch_xq_many_ring<NB, false>(tb, blocks, st);
    return launch_xq_many_ring<NB, true>(tb, blocks, st);
}

hipError_t launch_xq_bf16_many(const XqArgs* a, int n, hipStream_t st) {
    if (n < 0 || n > kBatchMax) return hipErrorInvalidValue;
    KBatch<XqDev> tb, fin;
    tb.n = fin.n = 0;
    uint64_t blocks = 0, fin_blocks = 0;
    int rp = 0;
    for (int m = 0; m < n; ++m) {
        if (a[m].M == 0) continue;
        if (rp == 0) rp = a[m].rp;
        if (a[m].rp != rp) return hipErrorInvalidValue;       // one padded rank per launch
        XqDev d;
        d.X = a[m].X; d.ldx = a[m].ldx; d.M = a[m].M; d.K = a[m].K; d.Qpack = a[m].Qpack; d.r = a[m].r;
        d.T = a[m].T; d.TpackT = a[m].TpackT; d.m_pad = a[m].m_pad;
        d.rows = a[m].TpackT ? a[m].m_pad : a[m].M;
        d.ns = a[m].part ? xq_splits(a[m].m_pad, a[m].K) : 1;
        d.part = d.ns > 1 ? a[m].part : nullptr;
        const uint32_t gx = (uint32_t)((d.rows + XQ_TOK - 1) / XQ_TOK);
        tb.first[tb.n] = (uint32_t)blocks; tb.gx[tb.n] = gx; tb.a[tb.n++] = d;
        blocks += (uint64_t)gx * (uint32_t)d.ns;
        if (d.ns > 1) {
            const uint32_t fx = (uint32_t)((d.rows * rp + 255) / 256);
            fin.first[fin.n] = (uint32_t)fin_blocks; fin.gx[fin.n] = fx; fin.a[fin.n++] = d;
            fin_blocks += fx;
        }
    }
    if (tb.n == 0) return hipSuccess;
    if (blocks > 0x7FFFFFFFull || fin_blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipError_t e;
    switch (rp / 16) {
        case 1: e = launch_xq_many_nb<1>(tb, (unsigned)blocks, st); break;
        case 2: e = launch_xq_many_nb<2>(tb, (unsigned)blocks, st); break;
        case 3: e = launch_xq_many_nb<3>(tb, (unsigned)blocks, st); break;
        case 4: e = launch_xq_many_nb<4>(tb, (unsigned)blocks, st); break;
        default: return hipErrorInvalidValue;
    }
    if (e != hipSuccess || fin.n == 0) return e;
    hipLaunchKernelGGL(xq_finish_many_kernel, dim3((unsigned)fin_blocks), dim3(256), 0, st, fin, rp);
    return hipGetLastError();
}

hipError_t launch_xq_bf16(const bf16_t* X, int64_t ldx, int64_t M, int64_t K, const bf16_t* Qpack, int r, int rp,
                          float* T, bf16_t* TpackT, int64_t m_pad, float* part, hipStream_t st) {
    if (M == 0) return hipSuccess;
    // cover the padded token range too so that the planes' tail is zeroed
    const int64_t rows = TpackT ? m_pad : M;
    // the split is sized for the padded range, which is what the workspace was sized for
    const int ns = part ? xq_splits(m_pad, K) : 1;
    dim3 grid((unsigned)((rows + XQ_TOK - 1) / XQ_TOK), (unsigned)ns);
    float* p = ns > 1 ? part : nullptr;
    hipError_t e;
    switch (rp / 16) {
        case 1: e = launch_xq_nb<1>(grid, st, X, ldx, M, K, Qpack, r, T, TpackT, m_pad, p); break;
        case 2: e = launch_xq_nb<2>(grid, st, X, ldx, M, K, Qpack, r, T, TpackT, m_pad, p); break;
        case 3: e = launch_xq_nb<3>(grid, st, X, ldx, M, K, Qpack, r, T, TpackT, m_pad, p); break;
        case 4: e = launch_xq_nb<4>(grid, st, X, ldx, M, K, Qpack, r, T, TpackT, m_pad, p); break;
        default: return hipErrorInvalidValue;
    }
    if (e != hipSuccess || ns == 1) return e;
    const int64_t items = rows * rp;
    hipLaunchKernelGGL(xq_finish_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, st, p, ns, rows, M, m_pad, r, rp, T, TpackT);
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
    // at least about one workgroup per CU; with many tokens up to eight token ranges even when the panels alone fill
    // the chip (activations wider than the last-level cache come from HBM and need the bytes in flight: 814 -> 696 us
    // per extraction at 16384 x 12288); more ranges than that cost more in partial sums than they hide
    int64_t want = (256 + panels - 1) / panels;
    const int64_t by_tokens = M / 1024 < 8 ? M / 1024 : 8;
    if (want < by_tokens) want = by_tokens;
    const int64_t max_splits = (M + 4 * XTT_STEP - 1) / (4 * XTT_STEP);
    if (want > max_splits) want = max_splits;
    if (want < 1) want = 1;
    if (want > 16) want = 16;
    return (int)want;
}

// bx: panel of features, by: token range
template <int NB>
__device__ __forceinline__ void xtt_bf16_body(const bf16_t* __restrict__ X, int64_t ldx, int64_t M, int64_t K,
                                              const bf16_t* __restrict__ TpackT, int64_t m_pad,
                                              float* __restrict__ partial, int64_t tok_per_split, uint32_t bx, uint32_t by) {
    constexpr int RP = NB * 16;
    extern __shared__ __align__(16) float sbuf[];   // [XTT_PANEL][RP]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lc = lane & 15, lg = lane >> 4;
    const int64_t db = (int64_t)bx * XTT_PANEL;
    const int split = (int)by;
    const int64_t ts = (int64_t)split * tok_per_split;
    const int64_t te = min(ts + tok_per_split, m_pad);

    floatx4 acc[NB][8];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[nb][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    const int64_t dcol = db + lc * 8;
    const bool din = dcol < K;
    // one 32-token step: 8 KB of X and the T planes per wave.  The next step's loads are issued before this step's
    // matrix work (twice the bytes in flight: with one step in flight the sweep ran at memory latency); they are
    // unconditional, the step after the last one re-reads the last (clamped) and is dropped.
    auto load_step = [&](int64_t tb, uint4 (&v)[8], Frag (&a)[NB][3]) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int64_t t = min(tb + lg * 8 + i, M - 1);   // rows past M meet zero planes
            v[i] = din ? *reinterpret_cast<const uint4*>(X + t * ldx + dcol) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int pl = 0; pl < 3; ++pl)
                a[nb][pl].u = *reinterpret_cast<const uint4*>(TpackT + ((int64_t)(pl * RP + nb * 16 + lc)) * m_pad + tb + lg * 8);
    };
    int64_t tb = ts + wave * XTT_STEP;
    if (tb < te) {
        uint4 v[8];
        Frag a[NB][3];
        load_step(tb, v, a);
        for (; tb < te; tb += 4 * XTT_STEP) {
            uint4 vn[8];
            Frag an[NB][3];
            load_step(min(tb + 4 * XTT_STEP, te - XTT_STEP), vn, an);
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
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = vn[i];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int pl = 0; pl < 3; ++pl) a[nb][pl] = an[nb][pl];
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

template <int NB>
__global__ __launch_bounds__(256) void xtt_bf16_kernel(const bf16_t* __restrict__ X, int64_t ldx, int64_t M, int64_t K,
                                                       const bf16_t* __restrict__ TpackT, int64_t m_pad,
                                                       float* __restrict__ partial, int64_t tok_per_split) {
    xtt_bf16_body<NB>(X, ldx, M, K, TpackT, m_pad, partial, tok_per_split, blockIdx.x, blockIdx.y);
}

struct XttDev {
    const bf16_t* X; int64_t ldx, M, K;
    const bf16_t* TpackT; int64_t m_pad;
    float* partial; int64_t tok_per_split;
};
template <int NB>
__global__ __launch_bounds__(256) void xtt_bf16_many_kernel(const KBatch<XttDev> tb) {
    uint32_t bx, by;
    const XttDev& a = tb.a[kbatch_find(tb, bx, by)];
    xtt_bf16_body<NB>(a.X, a.ldx, a.M, a.K, a.TpackT, a.m_pad, a.partial, a.tok_per_split, bx, by);
}

static int64_t xtt_tokens_per_split(int64_t m_pad, int nsplit) {
    const int64_t t = (m_pad + nsplit - 1) / nsplit;
    return (t + 4 * XTT_STEP - 1) / (4 * XTT_STEP) * (4 * XTT_STEP);
}

hipError_t launch_xtt_bf16_many(const XttArgs* a, int n, hipStream_t st) {
    if (n < 0 || n > kBatchMax) return hipErrorInvalidValue;
    KBatch<XttDev> tb;
    tb.n = 0;
    uint64_t blocks = 0;
    int rp = 0;
    for (int m = 0; m < n; ++m) {
        if (a[m].M == 0 || a[m].K == 0) continue;
        if (rp == 0) rp = a[m].rp;
        if (a[m].rp != rp || a[m].nsplit < 1) return hipErrorInvalidValue;
        XttDev d;
        d.X = a[m].X; d.ldx = a[m].ldx; d.M = a[m].M; d.K = a[m].K; d.TpackT = a[m].TpackT; d.m_pad = a[m].m_pad;
        d.partial = a[m].partial; d.tok_per_split = xtt_tokens_per_split(a[m].m_pad, a[m].nsplit);
        const uint32_t gx = (uint32_t)((a[m].K + XTT_PANEL - 1) / XTT_PANEL);
        tb.first[tb.n] = (uint32_t)blocks; tb.gx[tb.n] = gx; tb.a[tb.n++] = d;
        blocks += (uint64_t)gx * (uint32_t)a[m].nsplit;
    }
    if (tb.n == 0) return hipSuccess;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const size_t smem = (size_t)XTT_PANEL * rp * sizeof(float);
    const dim3 grid((unsigned)blocks);
    switch (rp / 16) {
        case 1: hipLaunchKernelGGL(xtt_bf16_many_kernel<1>, grid, dim3(256), smem, st, tb); break;
        case 2: hipLaunchKernelGGL(xtt_bf16_many_kernel<2>, grid, dim3(256), smem, st, tb); break;
        case 3: hipLaunchKernelGGL(xtt_bf16_many_kernel<3>, grid, dim3(256), smem, st, tb); break;
        case 4: hipLaunchKernelGGL(xtt_bf16_many_kernel<4>, grid, dim3(256), smem, st, tb); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_xtt_bf16(const bf16_t* X, int64_t ldx, int64_t M, int64_t K, const bf16_t* TpackT, int64_t m_pad,
                           int rp, float* partial, int nsplit, hipStream_t st) {
    if (M == 0 || K == 0) return hipSuccess;
    const int64_t tok_per_split = xtt_tokens_per_split(m_pad, nsplit);
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
