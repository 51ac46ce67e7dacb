// Forward GEMM of the bf16 path for shapes that give too few 256 x 256 tiles to fill the chip (few tokens, narrow
// layers):  Y = X W^T (+ eps * (X B) G^T, Eq. 7) with fp32 accumulation, optional Y store and the squared-error loss of
// Sec. 4.1 from the accumulators.
//
// 128 x 128 tile per workgroup, 4 waves of 64 x 64 (2 x 2 blocks of v_mfma_f32_32x32x16_bf16), K slices of 64 double
// buffered in LDS (64 KiB per workgroup: two workgroups per compute unit).  Four times the workgroups of the large
// tiling, at twice its LDS reads per MFMA: the better trade while the large tiling would leave compute units idle.
// Operands travel global -> registers -> LDS (the next slice is in flight in registers while the current one is
// multiplied), in the same swizzled layout and with the same permutation of W rows as the large tiling, so a lane
// again ends up with one token and 16 consecutive outputs per block.  The rank-r term comes as extra K slices from
// the extension operands that gemm_ext_prep_kernel wrote ([Ph|Ph|Pl] against [Gh|Gl|Gh], eps folded in), appended
// after the d_in slices so that both signs share bit-identical X W^T accumulators.
//
// SK = true also emits the range sketch of Alg. 1 (first product, Y <- H Omega; here S = X^T Omega) from the X tiles
// that the forward stages in LDS anyway (Sec. 4.1: the pass that evaluates f0 also yields the layer's basis): tile
// (tm, tn) contracts its 128 tokens against Omega for the d_in slices tn, tn + tiles_n, ..., so that every slice of
// every token tile is sketched exactly once over the grid, and writes S's partial sum for that token tile
// (sk_partial[tm][d_in][16]; whoever consumes the sketch adds the token tiles in a fixed order).  Omega^T comes as the
// three bf16 planes of its fp32 values, token-contiguous, and is kept in LDS for the whole tile; the contraction runs
// over tokens while the X tile holds a token's features side by side, so a lane fetches one 32-bit word (two
// features) of eight tokens and a byte permute puts one feature's eight tokens side by side: wave w takes word w of
// every 16-byte chunk, lanes 0-7 of a 16-lane group its low half and lanes 8-15 its high half, which makes one
// 16 x 16 x 32 matrix instruction cover the wave's 16 features of the slice without idle columns.
#include "gemm_bf16_common.h"

namespace agzo {

constexpr int ST = BT_SMALL;                    // tile edge
constexpr int STILE_BYTES = ST * BK * 2;        // one operand tile: 16 KiB
constexpr int SMALL_SMEM = 4 * STILE_BYTES;      // 64 KiB: two operand tiles x two stages (the loss reduction reuses them)
constexpr int SK_RP = 16;                        // sketch columns of the fused range sketch (r <= 16)
constexpr int SK_ROW = ST * 2 + 16;              // bytes per row of the Omega^T planes in LDS (padded against bank conflicts)
constexpr int SK_SMEM = 3 * SK_RP * SK_ROW;      // 12.75 KiB: two workgroups still share a compute unit

// (LDS allows two workgroups per compute unit = two waves per SIMD, so each wave may use half the register file)
template <bool SK>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void gemm_bf16_small_kernel(GemmParams p) {
    extern __shared__ __align__(16) char smem[];
    char* const Ts = smem + SMALL_SMEM;                       // SK: Omega^T planes [3][16][128 tokens] of this token tile
    auto Xs = [&](int buf) -> char* { return smem + buf * (2 * STILE_BYTES); };
    auto Ws = [&](int buf) -> char* { return smem + buf * (2 * STILE_BYTES) + STILE_BYTES; };
    double* red = reinterpret_cast<double*>(smem);           // used after the slice loop, when the operand buffers are idle

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (p.clk && blockIdx.x == 0 && tid == 0) { p.clk[0] = __builtin_readcyclecounter(); p.clk[1] = wall_clock64(); }
    const int wa = wave >> 1, wb = wave & 1;                 // wa splits the outputs, wb the tokens
    const int lr = lane & 31, lh = lane >> 5;

    // workgroup -> tile: groups of 8 token tiles per output tile, so that neighbours share a W tile and a band of X
    const int wg = (int)blockIdx.x;
    constexpr int GM = 8;
    const int group = wg / (GM * p.tiles_n);
    const int first_m = group * GM;
    const int gsz = min(GM, p.tiles_m - first_m);
    const int in_group = wg - group * GM * p.tiles_n;
    const int64_t tm = first_m + in_group % gsz, tn = in_group / gsz;
    const int64_t m0 = tm * ST, n0 = tn * ST;

    const int nd = (int)((p.K + BK - 1) / BK);               // slices of d_in (the last one may be ragged)
    const int next = (p.Xext != nullptr) ? p.ext_ld / BK : 0;
    const int total = nd + next;

    // staging: 1024 16-byte chunks per operand and slice, four per thread.  Rows past the end of a matrix are
    // clamped to its last row (they only feed outputs that the epilogue masks); chunks past the width are zero.
    constexpr int DEPTH = 4;                                 // slices in flight in registers
    uint4 rx[DEPTH][4], rw[DEPTH][4];
    uint32_t keep[DEPTH];                                    // all ones, or zero for a chunk past the operand's width
    int grow_x[4], grow_w[4], soff[4];                       // global row of this thread's chunks, LDS byte offset
    const int ccol = (tid & 7) * 8;                          // first column of the chunk inside a slice (same for all four)
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int idx = tid + 256 * t, row = idx >> 3, c = idx & 7;
        grow_x[t] = (int)min(m0 + row, p.M - 1);
        grow_w[t] = (int)min(n0 + (row & ~31) + w_perm(row & 31), p.N - 1);
        soff[t] = lds_off(row, c);
    }
    auto gload = [&](auto SET, int it) __attribute__((always_inline)) {
        constexpr int set = decltype(SET)::value;
        // a slice of X and W, or (past the d_in slices) of the extension operands: same rows, other base and stride
        const bool e = it >= nd;
        const int64_t k0 = (int64_t)(e ? it - nd : it) * BK + ccol;
        const int64_t width = e ? p.ext_ld : p.K;
        const bf16_t* xb = e ? p.Xext : p.X;
        const bf16_t* wbp = e ? p.Wext : p.W;
        const int64_t sx = e ? p.ext_ld : p.ldx, sw = e ? p.ext_ld : p.ldw;
        // every thread always loads (a chunk past the width re-reads column 0 and is zeroed on its way into LDS):
        // loads under a per-thread branch would make the number of loads in flight unknown to the compiler, which
        // then waits for all of them before the first LDS write and the prefetch depth is lost; so would touching
        // the loaded registers here
        const bool in = k0 < width;
        const int64_t kc = in ? k0 : 0;
        keep[set] = in ? 0xFFFFFFFFu : 0u;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            rx[set][t] = *reinterpret_cast<const uint4*>(xb + grow_x[t] * sx + kc);
            rw[set][t] = *reinterpret_cast<const uint4*>(wbp + grow_w[t] * sw + kc);
        }
    };
    auto sstore = [&](auto SET, int buf) __attribute__((always_inline)) {
        constexpr int set = decltype(SET)::value;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const uint32_t m = keep[set];
            *reinterpret_cast<uint4*>(Xs(buf) + soff[t]) = make_uint4(rx[set][t].x & m, rx[set][t].y & m, rx[set][t].z & m, rx[set][t].w & m);
            *reinterpret_cast<uint4*>(Ws(buf) + soff[t]) = make_uint4(rw[set][t].x & m, rw[set][t].y & m, rw[set][t].z & m, rw[set][t].w & m);
        }
    };

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    auto multiply = [&](int buf) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8 a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) a[i] = *reinterpret_cast<const bf16x8*>(Ws(buf) + lds_off(wa * 64 + i * 32 + lr, kk * 2 + lh));
#pragma unroll
            for (int j = 0; j < 2; ++j) b[j] = *reinterpret_cast<const bf16x8*>(Xs(buf) + lds_off(wb * 64 + j * 32 + lr, kk * 2 + lh));
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    };

    // ---- fused range sketch (SK) ----
    int sk_next = (int)tn;                                   // next slice this tile sketches
    if (SK) {
        // planes [pl][k][m0 .. m0 + 127] -> LDS: 768 16-byte chunks (sk_mpad covers whole 128-token tiles)
        for (int idx = tid; idx < 3 * SK_RP * (ST / 8); idx += 256) {
            const int row = idx / (ST / 8), ch = idx % (ST / 8);
            *reinterpret_cast<uint4*>(Ts + row * SK_ROW + ch * 16) =
                *reinterpret_cast<const uint4*>(p.sk_T + (int64_t)row * p.sk_mpad + m0 + ch * 8);
        }
    }
    auto sketch = [&](int buf, int it) __attribute__((always_inline)) {
        typedef float f32x4 __attribute__((ext_vector_type(4)));
        // (lane roles are recomputed here and the token chunks are not unrolled: the slice loop has no registers to spare)
        const int sk_n = lane & 15, sk_g = lane >> 4, sk_c = sk_n & 7;
        const uint32_t sk_sel = (sk_n >> 3) ? 0x07060302u : 0x05040100u;
        f32x4 sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
        for (int tc = 0; tc < 4; ++tc) {
            uint32_t wv[8];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                wv[i] = *reinterpret_cast<const uint32_t*>(Xs(buf) + lds_off(32 * tc + 8 * sk_g + i, sk_c) + 4 * wave);
            union { uint4 u; bf16x8 v; } b, a;
            b.u = make_uint4(__builtin_amdgcn_perm(wv[1], wv[0], sk_sel), __builtin_amdgcn_perm(wv[3], wv[2], sk_sel),
                             __builtin_amdgcn_perm(wv[5], wv[4], sk_sel), __builtin_amdgcn_perm(wv[7], wv[6], sk_sel));
#pragma unroll
            for (int pl = 0; pl < 3; ++pl) {
                a.u = *reinterpret_cast<const uint4*>(Ts + (pl * SK_RP + sk_n) * SK_ROW + (32 * tc + 8 * sk_g) * 2);
                sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, b.v, sacc, 0, 0, 0);
            }
        }
        // lane: feature = column sk_n of the block, sketch columns 4 sk_g .. 4 sk_g + 3
        const int64_t f = (int64_t)it * BK + 8 * sk_c + 2 * wave + (sk_n >> 3);
        if (f < p.K)
            *reinterpret_cast<float4*>(p.sk_partial + ((int64_t)tm * p.K + f) * SK_RP + 4 * sk_g) = make_float4(sacc[0], sacc[1], sacc[2], sacc[3]);
    };

    // Slice j travels through register set j % DEPTH: requested DEPTH iterations before it is multiplied (a single
    // slice in flight leaves the loop bound by memory latency: a 128 x 128 slice multiplies in a quarter of a
    // microsecond), written to LDS buffer j % 2 one iteration before.  The loop is unrolled by DEPTH so that the set
    // indices are compile-time constants.
    auto step = [&](auto U, int it) __attribute__((always_inline)) {
        constexpr int u = decltype(U)::value;                // it % DEPTH == u
        if (it + DEPTH < total) gload(IC<u>{}, it + DEPTH);  // set u held slice `it`, which is in LDS already
        multiply(it & 1);
        if (it + 1 < total) sstore(IC<(u + 1) % DEPTH>{}, (it + 1) & 1);    // the buffer that slice it-1 was read from
        if (SK && it == sk_next && it < nd) { sketch(it & 1, it); sk_next += p.tiles_n; }
        __syncthreads();
    };
    // the same without the tests, for the steady state: with nothing conditional between a request and its use the
    // compiler can count the loads in flight and waits only for the set it is about to write to LDS
    auto step_steady = [&](auto U, int it) __attribute__((always_inline)) {
        constexpr int u = decltype(U)::value;
        gload(IC<u>{}, it + DEPTH);
        multiply(it & 1);
        sstore(IC<(u + 1) % DEPTH>{}, (it + 1) & 1);
        if (SK && it == sk_next && it < nd) { sketch(it & 1, it); sk_next += p.tiles_n; }
        __syncthreads();
    };
    if (total > 0) {
        gload(IC<0>{}, 0);
        if (1 < total) gload(IC<1>{}, 1);
        if (2 < total) gload(IC<2>{}, 2);
        if (3 < total) gload(IC<3>{}, 3);
        sstore(IC<0>{}, 0);
        __syncthreads();
        int it = 0;
        for (; it + 2 * DEPTH <= total; it += DEPTH) {       // every step of the group has a slice to request
            step_steady(IC<0>{}, it);
            step_steady(IC<1>{}, it + 1);
            step_steady(IC<2>{}, it + 2);
            step_steady(IC<3>{}, it + 3);
        }
        for (; it < total; it += DEPTH) {                    // the last one or two groups
            step(IC<0>{}, it);
            if (it + 1 < total) step(IC<1>{}, it + 1);
            if (it + 2 < total) step(IC<2>{}, it + 2);
            if (it + 3 < total) step(IC<3>{}, it + 3);
        }
    }

    // ---- epilogue: lane = one token, 16 consecutive outputs per block ----
    const bool y_f32 = (p.Y != nullptr) && p.y_dtype != AGZO_BF16;
    const bool y_bf16 = (p.Y != nullptr) && p.y_dtype == AGZO_BF16;
    const bool l_f32 = p.loss_kind == AGZO_LOSS_MSE && p.target_dtype != AGZO_BF16;
    const bool l_bf16 = p.loss_kind == AGZO_LOSS_MSE && p.target_dtype == AGZO_BF16;
    double part = 0.0;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int64_t row = m0 + wb * 64 + j * 32 + lr;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int64_t col0 = n0 + wa * 64 + i * 32 + lh * 16;
            const floatx16 v = acc[i][j];
            if (row >= p.M || col0 >= p.N) continue;
            if (p.vec_ok && col0 + 16 <= p.N) {
                if (y_f32) {
                    float4* dst = reinterpret_cast<float4*>(reinterpret_cast<float*>(p.Y) + row * p.ldy + col0);
#pragma unroll
                    for (int q = 0; q < 4; ++q) dst[q] = make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
                }
                if (y_bf16) {
                    uint4* dst = reinterpret_cast<uint4*>(reinterpret_cast<bf16_t*>(p.Y) + row * p.ldy + col0);
                    uint32_t w[8];
#pragma unroll
                    for (int q = 0; q < 8; ++q) w[q] = pack_bf16x2(v[2 * q], v[2 * q + 1]);
                    dst[0] = make_uint4(w[0], w[1], w[2], w[3]);
                    dst[1] = make_uint4(w[4], w[5], w[6], w[7]);
                }
                // differences and squares in fp32, four at a time, summed in fp64 (as in the large tiling)
                if (l_f32) {
                    const uint4* src = reinterpret_cast<const uint4*>(reinterpret_cast<const float*>(p.target) + row * p.ldt + col0);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const uint4 t = src[q];
                        const float tv[4] = {__uint_as_float(t.x), __uint_as_float(t.y), __uint_as_float(t.z), __uint_as_float(t.w)};
                        float s4 = 0.f;
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            const float dd = v[4 * q + u] - tv[u];
                            s4 = fmaf(dd, dd, s4);
                        }
                        part += (double)s4;
                    }
                }
                if (l_bf16) {
                    const uint4* src = reinterpret_cast<const uint4*>(reinterpret_cast<const bf16_t*>(p.target) + row * p.ldt + col0);
#pragma unroll
                    for (int q = 0; q < 2; ++q) {
                        const uint4 t = src[q];
                        const uint32_t tw[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
                        for (int h = 0; h < 2; ++h) {
                            float s4 = 0.f;
#pragma unroll
                            for (int u = 0; u < 2; ++u) {
                                const uint32_t w = tw[2 * h + u];
                                const float d0 = v[8 * q + 4 * h + 2 * u] - __uint_as_float(w << 16);
                                const float d1 = v[8 * q + 4 * h + 2 * u + 1] - __uint_as_float(w & 0xFFFF0000u);
                                s4 = fmaf(d0, d0, s4);
                                s4 = fmaf(d1, d1, s4);
                            }
                            part += (double)s4;
                        }
                    }
                }
            } else {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int64_t col = col0 + e;
                    if (col < p.N) {
                        const float y = v[e];
                        if (y_f32) reinterpret_cast<float*>(p.Y)[row * p.ldy + col] = y;
                        if (y_bf16) reinterpret_cast<bf16_t*>(p.Y)[row * p.ldy + col] = f32_to_bf16(y);
                        float tv = 0.f;
                        if (l_f32) tv = reinterpret_cast<const float*>(p.target)[row * p.ldt + col];
                        if (l_bf16) tv = bf16_to_f32(reinterpret_cast<const bf16_t*>(p.target)[row * p.ldt + col]);
                        if (l_f32 || l_bf16) {
                            const float dd = y - tv;
                            part += (double)dd * (double)dd;
                        }
                    }
                }
            }
        }
    }
    if (p.loss_kind == AGZO_LOSS_MSE) {
        // the operand buffers are no longer read (barrier at the end of the slice loop), so red may lie in them
        red[tid] = part;
        __syncthreads();
        for (int s = 128; s > 0; s >>= 1) {
            if (tid < s) red[tid] += red[tid + s];
            __syncthreads();
        }
        if (tid == 0) p.partials[tm * p.tiles_n + tn] = red[0];
    }
    if (p.clk && blockIdx.x == 0 && tid == 0) { p.clk[2] = __builtin_readcyclecounter(); p.clk[3] = wall_clock64(); }
}

// p.tiles_m / p.tiles_n count 128 x 128 tiles here
hipError_t launch_gemm_bf16_small(const GemmParams& p, hipStream_t st) {
    dim3 grid((unsigned)((int64_t)p.tiles_m * p.tiles_n));
    if (p.sk_T) {
        // the sketch is taken from the d_in slices (at least one), for r <= 16
        if (!p.sk_partial || p.K < 1 || p.sk_mpad < (int64_t)p.tiles_m * ST) return hipErrorInvalidValue;
        static bool attr_set = false;
        if (!attr_set) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_bf16_small_kernel<true>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, SMALL_SMEM + SK_SMEM);
            if (e != hipSuccess) return e;
            attr_set = true;
        }
        hipLaunchKernelGGL(gemm_bf16_small_kernel<true>, grid, dim3(256), SMALL_SMEM + SK_SMEM, st, p);
    } else {
        hipLaunchKernelGGL(gemm_bf16_small_kernel<false>, grid, dim3(256), SMALL_SMEM, st, p);
    }
    return hipGetLastError();
}

}  // namespace agzo
