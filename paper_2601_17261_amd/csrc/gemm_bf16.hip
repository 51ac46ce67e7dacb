// Forward GEMM of the bf16 path on the CDNA4 matrix cores:
//     Y = X W^T  (+ eps * (X B) G^T, the factored form of Eq. 7)   with fp32 accumulation,
// and the loss of Sec. 4.1 (f0, f+, f-) reduced from the fp32 accumulators in the epilogue.
//
// Tiling: one workgroup (256 threads = 4 wave64) owns a 256 x 256 tile of Y; each wave owns a
// 128 x 128 quadrant as 4 x 4 blocks of v_mfma_f32_32x32x16_bf16.  X and W are both K-contiguous
// (an "NT" product), staged through LDS in 64-wide K slices, double buffered.
// The rank-r term is accumulated by the same MFMA loop as a few extra K slices appended after
// the d_in slices: A-operand = eps * P split in bf16 hi/lo, B-operand = G regenerated from the
// Philox seed and split likewise, so both signs share bit-identical X W^T accumulators.
#include "agzo_internal.h"

namespace agzo {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int CHUNKS = BK / 8;                 // 16-byte chunks per tile row
constexpr int TILE_BYTES = BM * BK * 2;        // one operand tile: 32 KiB

int gemm_bf16_num_workgroups(int64_t M, int64_t N) {
    return (int)(((M + BM - 1) / BM) * ((N + BN - 1) / BN));
}

// byte offset of 16-byte chunk `c` of row `row` inside a [256][64] bf16 tile; the XOR spreads the
// rows of one MFMA operand read over all LDS banks.
__device__ __forceinline__ int lds_off(int row, int c) { return row * (BK * 2) + ((c ^ ((row >> 1) & 7)) << 4); }

struct GemmParams {
    const bf16_t* X; int64_t ldx;
    const bf16_t* W; int64_t ldw;
    int64_t M, N, K;
    void* Y; int y_dtype; int64_t ldy;
    const float* P; int r; int rp;
    float eps_signed; uint32_t s_lo, s_hi;
    int loss_kind; int target_dtype; const void* target; int64_t ldt; double* partials;
    int tiles_m, tiles_n;
};

__device__ __forceinline__ void compute_tile(const char* As, const char* Bs, int wm, int wn, int lane,
                                             floatx16 (&acc)[4][4]) {
    const int lr = lane & 31, lh = lane >> 5;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
        bf16x8 a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            a[i] = *reinterpret_cast<const bf16x8*>(As + lds_off(wm * 128 + i * 32 + lr, kk * 2 + lh));
#pragma unroll
        for (int j = 0; j < 4; ++j)
            b[j] = *reinterpret_cast<const bf16x8*>(Bs + lds_off(wn * 128 + j * 32 + lr, kk * 2 + lh));
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
}

__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmParams p) {
    extern __shared__ __align__(16) char smem[];
    auto As = [&](int buf) -> char* { return smem + buf * (2 * TILE_BYTES); };
    auto Bs = [&](int buf) -> char* { return smem + buf * (2 * TILE_BYTES) + TILE_BYTES; };

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // workgroup -> tile: consecutive ids of one XCD (ids are dealt round-robin over the 8 XCDs)
    // walk down a column of tiles, so an XCD's L2 keeps a W tile and streams X tiles under it.
    int64_t wg = blockIdx.x;
    const int64_t nwg = (int64_t)p.tiles_m * p.tiles_n;
    {
        const int64_t per = nwg / 8;
        if (wg < per * 8) wg = (wg % 8) * per + wg / 8;
    }
    constexpr int GROUP_M = 8;
    const int64_t group = wg / (GROUP_M * p.tiles_n);
    const int64_t first_m = group * GROUP_M;
    const int gsz = (int)min((int64_t)GROUP_M, p.tiles_m - first_m);
    const int64_t in_group = wg - group * GROUP_M * p.tiles_n;
    const int64_t tm = first_m + in_group % gsz;
    const int64_t tn = in_group / gsz;
    const int64_t m0 = tm * BM, n0 = tn * BN;

    floatx16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // global -> LDS staging: thread owns chunk (tid % 8) of rows tid/8 + 32*i
    const int lc = tid & 7;
    const int lrow = tid >> 3;
    uint4 ra[8], rb[8];
    const int64_t nk = (p.K + BK - 1) / BK;

    auto gload = [&](int64_t kt) {
        const int64_t kcol = kt * BK + lc * 8;
        const bool kin = kcol < p.K;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = lrow + 32 * i;
            int64_t gm = min(m0 + row, p.M - 1);
            int64_t gn = min(n0 + row, p.N - 1);
            ra[i] = kin ? *reinterpret_cast<const uint4*>(p.X + gm * p.ldx + kcol) : make_uint4(0, 0, 0, 0);
            rb[i] = kin ? *reinterpret_cast<const uint4*>(p.W + gn * p.ldw + kcol) : make_uint4(0, 0, 0, 0);
        }
    };
    auto lstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = lrow + 32 * i;
            *reinterpret_cast<uint4*>(As(buf) + lds_off(row, lc)) = ra[i];
            *reinterpret_cast<uint4*>(Bs(buf) + lds_off(row, lc)) = rb[i];
        }
    };

    gload(0);
    lstore(0);
    __syncthreads();
    for (int64_t kt = 0; kt < nk; ++kt) {
        const int cur = (int)(kt & 1);
        if (kt + 1 < nk) gload(kt + 1);
        compute_tile(As(cur), Bs(cur), wm, wn, lane, acc);
        if (kt + 1 < nk) lstore(cur ^ 1);
        __syncthreads();
    }

    // ---- rank-r term: extra K slices [Ph|Ph|Pl] x [Gh|Gl|Gh] --------------------------------
    if (p.P != nullptr) {
        const int rp = p.rp;                  // r rounded up to 16
        const int kext = 3 * rp;              // columns of the extended operands
        const int next = (kext + BK - 1) / BK;
        const int kchunks = rp / 8;           // 8-column chunks of P' and G per row
        for (int et = 0; et < next; ++et) {
            // chunks of this slice that lie beyond the extended width are zero
            for (int e = tid; e < BM * CHUNKS; e += 256) {
                const int row = e >> 3, c = e & 7;
                if (et * BK + c * 8 >= kext) {
                    *reinterpret_cast<uint4*>(As(0) + lds_off(row, c)) = make_uint4(0, 0, 0, 0);
                    *reinterpret_cast<uint4*>(Bs(0) + lds_off(row, c)) = make_uint4(0, 0, 0, 0);
                }
            }
            // one item = 8 consecutive k of one tile row: P' (for X row m0+row) and G (for W row n0+row),
            // written to each of the three segments that falls into this slice
            for (int e = tid; e < BM * kchunks; e += 256) {
                const int row = e / kchunks, k0 = (e - row * kchunks) * 8;
                bool need = false;
#pragma unroll
                for (int seg = 0; seg < 3; ++seg) need |= ((seg * rp + k0) / BK == et);
                if (!need) continue;
                const int64_t gm = m0 + row, gn = n0 + row;
                float pv[8], gv[8];
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    pv[i] = (gm < p.M && k0 + i < p.r) ? p.eps_signed * p.P[gm * p.r + k0 + i] : 0.f;
                {
                    float4 z0 = make_float4(0.f, 0.f, 0.f, 0.f), z1 = z0;
                    if (gn < p.N) {
                        if (k0 < p.r) z0 = philox_normal4(p.s_lo, p.s_hi, AGZO_TAG_G, (uint32_t)gn, (uint32_t)(k0 >> 2));
                        if (k0 + 4 < p.r)
                            z1 = philox_normal4(p.s_lo, p.s_hi, AGZO_TAG_G, (uint32_t)gn, (uint32_t)((k0 >> 2) + 1));
                    }
                    const float t[8] = {z0.x, z0.y, z0.z, z0.w, z1.x, z1.y, z1.z, z1.w};
#pragma unroll
                    for (int i = 0; i < 8; ++i) gv[i] = (k0 + i < p.r) ? t[i] : 0.f;
                }
                uint32_t ph[4] = {0, 0, 0, 0}, pl[4] = {0, 0, 0, 0}, gh[4] = {0, 0, 0, 0}, gl[4] = {0, 0, 0, 0};
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const bf16_t a_hi = f32_to_bf16(pv[i]);
                    const bf16_t a_lo = f32_to_bf16(pv[i] - bf16_to_f32(a_hi));
                    const bf16_t b_hi = f32_to_bf16(gv[i]);
                    const bf16_t b_lo = f32_to_bf16(gv[i] - bf16_to_f32(b_hi));
                    const int sh = (i & 1) * 16;
                    ph[i >> 1] |= ((uint32_t)a_hi) << sh;
                    pl[i >> 1] |= ((uint32_t)a_lo) << sh;
                    gh[i >> 1] |= ((uint32_t)b_hi) << sh;
                    gl[i >> 1] |= ((uint32_t)b_lo) << sh;
                }
#pragma unroll
                for (int seg = 0; seg < 3; ++seg) {
                    const int col0 = seg * rp + k0;
                    if (col0 / BK != et) continue;
                    const int c = (col0 - et * BK) >> 3;
                    const uint32_t* av = (seg == 2) ? pl : ph;   // [Ph | Ph | Pl]
                    const uint32_t* bv = (seg == 1) ? gl : gh;   // [Gh | Gl | Gh]
                    *reinterpret_cast<uint4*>(As(0) + lds_off(row, c)) = make_uint4(av[0], av[1], av[2], av[3]);
                    *reinterpret_cast<uint4*>(Bs(0) + lds_off(row, c)) = make_uint4(bv[0], bv[1], bv[2], bv[3]);
                }
            }
            __syncthreads();
            compute_tile(As(0), Bs(0), wm, wn, lane, acc);
            __syncthreads();
        }
    }

    // ---- epilogue: optional store, loss partial ---------------------------------------------
    const int lr = lane & 31, lh = lane >> 5;
    double part = 0.0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t col = n0 + wn * 128 + j * 32 + lr;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int64_t row = m0 + wm * 128 + i * 32 + (e >> 2) * 8 + lh * 4 + (e & 3);
                if (row < p.M && col < p.N) {
                    const float y = acc[i][j][e];
                    if (p.Y != nullptr) {
                        if (p.y_dtype == AGZO_BF16)
                            reinterpret_cast<bf16_t*>(p.Y)[row * p.ldy + col] = f32_to_bf16(y);
                        else
                            reinterpret_cast<float*>(p.Y)[row * p.ldy + col] = y;
                    }
                    if (p.loss_kind == AGZO_LOSS_MSE) {
                        const float tv = (p.target_dtype == AGZO_BF16)
                                             ? bf16_to_f32(reinterpret_cast<const bf16_t*>(p.target)[row * p.ldt + col])
                                             : reinterpret_cast<const float*>(p.target)[row * p.ldt + col];
                        const double d = (double)y - (double)tv;
                        part = fma(d, d, part);
                    }
                }
            }
        }
    }
    if (p.loss_kind == AGZO_LOSS_MSE) {
        double* red = reinterpret_cast<double*>(smem);
        red[tid] = part;
        __syncthreads();
        for (int s = 128; s > 0; s >>= 1) {
            if (tid < s) red[tid] += red[tid + s];
            __syncthreads();
        }
        if (tid == 0) p.partials[tm * p.tiles_n + tn] = red[0];
    }
}

hipError_t launch_gemm_bf16(const GemmBf16Args& a, hipStream_t st) {
    if (a.M == 0 || a.N == 0) return hipSuccess;
    GemmParams p;
    p.X = a.X; p.ldx = a.ldx; p.W = a.W; p.ldw = a.ldw;
    p.M = a.M; p.N = a.N; p.K = a.K;
    p.Y = a.Y; p.y_dtype = a.y_dtype; p.ldy = a.ldy;
    p.P = a.P; p.r = a.r; p.rp = (a.r + 15) / 16 * 16;
    p.eps_signed = a.eps_signed; p.s_lo = (uint32_t)a.seed; p.s_hi = (uint32_t)(a.seed >> 32);
    p.loss_kind = a.loss.kind; p.target_dtype = a.loss.target_dtype; p.target = a.loss.target;
    p.ldt = a.loss.ldt; p.partials = a.loss.partials;
    p.tiles_m = (int)((a.M + BM - 1) / BM);
    p.tiles_n = (int)((a.N + BN - 1) / BN);
    static bool attr_set = false;
    const int smem = 4 * TILE_BYTES;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_bf16_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid((unsigned)((int64_t)p.tiles_m * p.tiles_n));
    hipLaunchKernelGGL(gemm_bf16_kernel, grid, dim3(256), smem, st, p);
    return hipGetLastError();
}

}  // namespace agzo
