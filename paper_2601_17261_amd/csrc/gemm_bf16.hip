// Forward GEMM of the bf16 path on the CDNA4 matrix cores:
//     Y = X W^T  (+ eps * (X B) G^T, the factored form of Eq. 7)   with fp32 accumulation,
// and the loss of Sec. 4.1 (f0, f+, f-) reduced from the fp32 accumulators in the epilogue.
//
// Tiling: one workgroup (4 waves, one per SIMD) owns a 256 (tokens) x 256 (outputs) tile of Y, one wave a
// 128 x 128 quarter: 16 accumulator blocks = 256 registers, which the compiler keeps in the accumulation half of
// the register file, leaving the other 256 for operands and the epilogue.  The large wave tile is what keeps the
// LDS traffic per MFMA low enough (8 fragment reads per 16 MFMAs).
// X and W are both K-contiguous (an "NT" product) and are staged through LDS in 64-wide K slices, double
// buffered, with direct global -> LDS loads.  MFMA roles (v_mfma_f32_32x32x16_bf16): A-operand = W rows,
// B-operand = X rows, so a lane owns one token and 16 output columns per 32x32 block; the W rows of a block are
// permuted on their way into LDS so that those 16 columns are consecutive and the epilogue moves 16-byte vectors.
// With one wave per SIMD nothing hides an issue stall, so the steady state is written in issue order: every MFMA
// is followed by at most one fragment read or one direct load, the 16 loads of the next slice are spread over
// three of the four 16-MFMA blocks, and the slice's barrier sits before its last block, whose MFMAs then cover
// the LDS latency of the next slice's first fragments.
// The rank-r term is accumulated by the same MFMA blocks as a few extra K slices appended after the d_in slices:
// one operand is eps * P split in bf16 hi/lo, the other is G regenerated from the Philox seed and split
// likewise, so both signs share bit-identical X W^T accumulators.
#include "gemm_bf16_common.h"

namespace agzo {

// true: the shape gives so few 256 x 256 tiles that most compute units would idle; the 128 x 128 tiling is used when
// the call is one it supports (no shared-forward mode, no cross-entropy)
static bool small_shape(int64_t M, int64_t N) {
    return ((M + BT - 1) / BT) * ((N + BT - 1) / BT) < 160;
}

bool gemm_bf16_fuses_sketch(int64_t M, int64_t N, int r, bool large_tiles) {
    return !large_tiles && small_shape(M, N) && r <= 16 && gemm_bf16_sketch_splits(M) <= 64;
}

int gemm_bf16_ce_chunks(int64_t N) { return (int)((N + BT - 1) / BT) * 2; }   // 128-column chunks (2 per tile)

int gemm_bf16_num_workgroups(int64_t M, int64_t N, bool small_ok) {
    if (small_ok && small_shape(M, N)) return (int)(((M + BT_SMALL - 1) / BT_SMALL) * ((N + BT_SMALL - 1) / BT_SMALL));
    return (int)(((M + BT - 1) / BT) * ((N + BT - 1) / BT));
}

// WA x WB waves: WA splits the 256 outputs, WB splits the 256 tokens
// EPI selects the epilogue compiled into the kernel: 0 = general (stores, squared error, any bounds), 1 = cross-entropy
// statistics.  (Tile-aligned layers with the squared-error loss and no stored Y, or a stored bf16 Y and no loss, take the kernel of
// gemm_bf16_aligned.hip.)
template <int WA, int WB, bool SHARED, int EPI>
__global__ __launch_bounds__(64 * WA * WB) void gemm_bf16_kernel(GemmParams p) {
    constexpr bool CE = (EPI == 1);
    constexpr int NT = 64 * WA * WB;
    constexpr int BA = BT / WA / 32;           // 32-row blocks of W per wave
    constexpr int BB = BT / WB / 32;           // 32-row blocks of X per wave
    extern __shared__ __align__(16) char smem[];
    auto Xs = [&](int buf) -> char* { return smem + buf * (2 * TILE_BYTES); };
    auto Ws = [&](int buf) -> char* { return smem + buf * (2 * TILE_BYTES) + TILE_BYTES; };

    const int tid = threadIdx.x, lane = tid & 63;
    if (p.clk && blockIdx.x == 0 && tid == 0) { p.clk[0] = __builtin_readcyclecounter(); p.clk[1] = wall_clock64(); }
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform by construction: keeps LDS bases scalar
    const int wa = wave / WB, wb = wave % WB;
    const int lr = lane & 31, lh = lane >> 5;

    // workgroup -> tile.  Ids are dealt round-robin over the 8 XCDs; give each XCD a contiguous
    // run of tiles, walked in groups of 8 token-tiles per output-tile so that its L2 keeps a W tile
    // and a band of X tiles.
    int wg = (int)blockIdx.x;
    const int nwg = p.tiles_m * p.tiles_n;
    {
        const int per = nwg / 8;
        if (wg < per * 8) wg = (wg % 8) * per + wg / 8;
    }
    const int GROUP_M = p.group_m;
    const int group = wg / (GROUP_M * p.tiles_n);
    const int first_m = group * GROUP_M;
    const int gsz = min(GROUP_M, p.tiles_m - first_m);
    const int in_group = wg - group * GROUP_M * p.tiles_n;
    // the divisions run on the vector unit; pin the (uniform) results to scalar registers so that everything derived
    // from the tile origin, the buffer descriptors above all, stays scalar
    const int64_t tm = __builtin_amdgcn_readfirstlane(first_m + in_group % gsz);
    const int64_t tn = __builtin_amdgcn_readfirstlane(in_group / gsz);
    const int64_t m0 = tm * BT, n0 = tn * BT;

    floatx16 acc[BA][BB];
#pragma unroll
    for (int i = 0; i < BA; ++i)
#pragma unroll
        for (int j = 0; j < BB; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // ---- operand staging ------------------------------------------------------------------------
    // Whole 64-wide K slices travel global -> LDS without passing through registers
    // (buffer_load_dwordx4 ... lds: lane l of a wave writes its 16 bytes at LDS base + 16*l, so one
    // instruction fills 8 consecutive tile rows).  The bank swizzle is applied on the global side by
    // choosing which 16-byte chunk of its row a lane fetches.  Slices that are not plain copies of
    // memory (the ragged end of d_in, the rank-r extension) are written by the threads themselves.
    static_assert(WA == 2 && WB == 2 && BA == 4 && BB == 4, "the issue schedule below is written for 2 x 2 waves");
    constexpr int GP = 8;                       // 8-row groups per wave per operand
    const bf16_t* xbase = p.X + m0 * p.ldx;
    const bf16_t* wbase = p.W + n0 * p.ldw;
    // Buffer descriptors with the tile's own byte range: rows past the end of the matrix are out of range for the
    // descriptor, so their loads fetch nothing (zeros) and no address has to be clamped; such rows only feed outputs
    // that the epilogue masks.  That makes the offset of row group t a scalar multiple of t: one vector offset per
    // operand instead of one per group.
    auto tile_rsrc = [&](const bf16_t* base, int64_t rows_left, int64_t ld, int64_t width) {
        // (a descriptor with a real range costs about 6 % of the load rate on this chip, so only the tiles that
        // hang over the edge get one)
        int64_t bytes = ((rows_left - 1) * ld + width) * 2;
        if (bytes > 0xFFFFFFFFll || rows_left >= BT) bytes = 0xFFFFFFFFll;
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(base), 0, (int)(uint32_t)bytes, 0x00020000);
    };
    const __amdgpu_buffer_rsrc_t rx = tile_rsrc(xbase, p.M - m0, p.ldx, p.K);
    const __amdgpu_buffer_rsrc_t rw = tile_rsrc(wbase, p.N - n0, p.ldw, p.K);
    const __amdgpu_buffer_rsrc_t rx2 = tile_rsrc(p.Xext ? p.Xext + m0 * p.ext_ld : xbase, p.M - m0, p.Xext ? p.ext_ld : p.ldx, p.Xext ? p.ext_ld : p.K);
    const __amdgpu_buffer_rsrc_t rw2 = tile_rsrc(p.Wext ? p.Wext + n0 * p.ext_ld : wbase, p.N - n0, p.Wext ? p.ext_ld : p.ldw, p.Wext ? p.ext_ld : p.K);
    const int row0 = 8 * wave + (lane >> 3);                 // row of group t = row0 + 32 t (X), 32 t + w_perm(row0) (W)
    const int chunk0 = (lane & 7) ^ ((row0 >> 1) & 7);       // (row >> 1) & 7 does not depend on t
    const int vx = (int)(((int64_t)row0 * p.ldx + chunk0 * 8) * 2), vw = (int)(((int64_t)w_perm(row0) * p.ldw + chunk0 * 8) * 2);
    const int vx2 = (row0 * p.ext_ld + chunk0 * 8) * 2, vw2 = (w_perm(row0) * p.ext_ld + chunk0 * 8) * 2;
    const int gsx = (int)(64 * p.ldx), gsw = (int)(64 * p.ldw), gs2 = 64 * p.ext_ld;   // bytes between row groups
    // the shared-forward variant addresses per lane (see dma1) and keeps clamped per-group offsets
    int xo[SHARED ? GP : 1], wo[SHARED ? GP : 1];
    if constexpr (SHARED) {
#pragma unroll
        for (int t = 0; t < GP; ++t) {
            const int row = 8 * (wave + 4 * t) + (lane >> 3);
            const int c = (lane & 7) ^ ((row >> 1) & 7);
            const int64_t gm = min((int64_t)row, p.M - 1 - m0);
            const int64_t gn = min((int64_t)((row & ~31) + w_perm(row & 31)), p.N - 1 - n0);
            xo[t] = (int)((gm * p.ldx + c * 8) * 2);
            wo[t] = (int)((gn * p.ldw + c * 8) * 2);
        }
    }
    const int nfull = (int)(p.K / BK);
    const int ntail = (p.K % BK) ? 1 : 0;
    const int rp = p.rp;                        // r rounded up to 16
    const int kext = 3 * rp;                    // width of the extended operands [Ph|Ph|Pl] x [Gh|Gl|Gh]
    const int next = (p.P != nullptr) ? (kext + BK - 1) / BK : 0;
    const int nd = nfull + ntail;               // slices of d_in
    // extension slices that come as ready-made operands ride the load pipeline right behind the plain slices
    const bool ext_dma = !SHARED && p.Xext != nullptr;
    const int npipe = nfull + (ext_dma ? next : 0);
    // shared mode: the extension runs twice, with +eps (accumulators become Y+) and then with -2 eps (Y-)
    const int total = nd + (SHARED ? 2 * next : next);

    // ragged last slice of d_in: chunks past d_in are zero
    auto fill_tail = [&](int buf) {
        for (int e = tid; e < BT * CHUNKS; e += NT) {
            const int row = e >> 3, c = e & 7;
            const int64_t kcol = (int64_t)nfull * BK + c * 8;
            uint4 vx = make_uint4(0, 0, 0, 0), vw = vx;
            if (kcol < p.K) {
                const int64_t gm = min((int64_t)row, p.M - 1 - m0);
                const int64_t gn = min((int64_t)((row & ~31) + w_perm(row & 31)), p.N - 1 - n0);
                vx = *reinterpret_cast<const uint4*>(xbase + gm * p.ldx + kcol);
                vw = *reinterpret_cast<const uint4*>(wbase + gn * p.ldw + kcol);
            }
            *reinterpret_cast<uint4*>(Xs(buf) + lds_off(row, c)) = vx;
            *reinterpret_cast<uint4*>(Ws(buf) + lds_off(row, c)) = vw;
        }
    };
    // slice `et` of the rank-r extension: X side eps*P as [hi|hi|lo], W side G as [hi|lo|hi]
    auto fill_ext = [&](int buf, int et, float coef) {
        const int kchunks = rp / 8;             // 8-column chunks of P' and G per row
        for (int e = tid; e < BT * CHUNKS; e += NT) {
            const int row = e >> 3, c = e & 7;
            if (et * BK + c * 8 >= kext) {      // beyond the extended width: zero
                *reinterpret_cast<uint4*>(Xs(buf) + lds_off(row, c)) = make_uint4(0, 0, 0, 0);
                *reinterpret_cast<uint4*>(Ws(buf) + lds_off(row, c)) = make_uint4(0, 0, 0, 0);
            }
        }
        // one item = 8 consecutive k of one tile row: P' for the token of X-tile row `row`, G for the
        // output held by W-tile row `row`; written to each segment that falls into this slice
        for (int e = tid; e < BT * kchunks; e += NT) {
            const int row = e / kchunks, k0 = (e - row * kchunks) * 8;
            bool need = false;
#pragma unroll
            for (int seg = 0; seg < 3; ++seg) need |= ((seg * rp + k0) / BK == et);
            if (!need) continue;
            const int64_t gm = m0 + row;
            const int64_t gn = n0 + (row & ~31) + w_perm(row & 31);
            float pv[8], gv[8];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                pv[i] = (gm < p.M && k0 + i < p.r) ? coef * p.P[gm * p.r + k0 + i] : 0.f;
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
            uint32_t ph[4], pl[4], gh[4], gl[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                ph[i] = pack_bf16x2(pv[2 * i], pv[2 * i + 1]);
                pl[i] = pack_bf16x2(pv[2 * i] - __uint_as_float(ph[i] << 16), pv[2 * i + 1] - __uint_as_float(ph[i] & 0xFFFF0000u));
                gh[i] = pack_bf16x2(gv[2 * i], gv[2 * i + 1]);
                gl[i] = pack_bf16x2(gv[2 * i] - __uint_as_float(gh[i] << 16), gv[2 * i + 1] - __uint_as_float(gh[i] & 0xFFFF0000u));
            }
#pragma unroll
            for (int seg = 0; seg < 3; ++seg) {
                const int col0 = seg * rp + k0;
                if (col0 / BK != et) continue;
                const int c = (col0 - et * BK) >> 3;
                const uint32_t* av = (seg == 2) ? pl : ph;   // [Ph | Ph | Pl]
                const uint32_t* bv = (seg == 1) ? gl : gh;   // [Gh | Gl | Gh]
                *reinterpret_cast<uint4*>(Xs(buf) + lds_off(row, c)) = make_uint4(av[0], av[1], av[2], av[3]);
                *reinterpret_cast<uint4*>(Ws(buf) + lds_off(row, c)) = make_uint4(bv[0], bv[1], bv[2], bv[3]);
            }
        }
    };
    auto fill_manual = [&](int it, int buf) {
        if (it < nd) {
            fill_tail(buf);
        } else {
            const int e = it - nd;
            if (SHARED && e >= next) fill_ext(buf, e - next, -2.f * p.eps_signed);
            else fill_ext(buf, e, p.eps_signed);
        }
    };
    typedef __attribute__((address_space(3))) void* lptr_t;

    double* red = reinterpret_cast<double*>(smem + 4 * TILE_BYTES);
    const bool y_f32 = (p.Y != nullptr) && p.y_dtype != AGZO_BF16;
    const bool y_bf16 = (p.Y != nullptr) && p.y_dtype == AGZO_BF16;
    const bool l_f32 = !CE && p.loss_kind == AGZO_LOSS_MSE && p.target_dtype != AGZO_BF16;
    const bool l_bf16 = !CE && p.loss_kind == AGZO_LOSS_MSE && p.target_dtype == AGZO_BF16;

    // ---- multiply ---------------------------------------------------------------------------------
    // per-lane LDS byte offsets of this wave's fragments for the four 16-wide sub-steps of a slice; block i of an
    // operand is 32 rows = 4096 bytes further (the swizzle term (row >> 1) & 7 is the same for all blocks)
    int aoff[4], boff[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        aoff[kk] = TILE_BYTES + lds_off(wa * 128 + lr, kk * 2 + lh);
        boff[kk] = lds_off(wb * 128 + lr, kk * 2 + lh);
    }
    bf16x8 a[2][BA], b[2][BB];
    auto frag1 = [&](int buf, int kk, int s, int q) __attribute__((always_inline)) {
        const char* base = smem + buf * (2 * TILE_BYTES);
        if (q < 4) a[s][q] = *reinterpret_cast<const bf16x8*>(base + aoff[kk] + q * 4096);
        else b[s][q - 4] = *reinterpret_cast<const bf16x8*>(base + boff[kk] + (q - 4) * 4096);
    };
    auto mfma1 = [&](int s, int idx) __attribute__((always_inline)) {
        const int i = idx >> 2, j = idx & 3;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s][i], b[s][j], acc[i][j], 0, 0, 0);
    };
    // Where a pipelined slice comes from: a plain 64-wide slice of X and W, or a slice of the ready-made extension
    // operands.  Chosen once per slice with scalar selects into one of two sets of variables (set 0: the slice loaded
    // by an iteration's first blocks, set 1: the one after it), so that the load sites themselves stay free of
    // branches, which would cut the fixed-order blocks below into pieces and put the accumulators through joins.
    __amdgpu_buffer_rsrc_t src_rsx[2] = {rx, rx}, src_rsw[2] = {rw, rw};
    int src_vx[2] = {vx, vx}, src_vw[2] = {vw, vw}, src_so[2] = {0, 0}, src_gx[2] = {gsx, gsx}, src_gw[2] = {gsw, gsw};
    auto select_slice = [&](auto SET, int kt) __attribute__((always_inline)) {
        constexpr int set = decltype(SET)::value;
        const bool e = kt >= nfull;
        src_rsx[set] = e ? rx2 : rx;   src_rsw[set] = e ? rw2 : rw;
        src_vx[set] = e ? vx2 : vx;    src_vw[set] = e ? vw2 : vw;
        src_so[set] = (e ? kt - nfull : kt) * (BK * 2);
        src_gx[set] = e ? gs2 : gsx;   src_gw[set] = e ? gs2 : gsw;
    };
    // direct load q (0..15) of the slice selected into SET, into buffer buf: even q = X row group q/2, odd q = W row group
    auto dma1 = [&](auto SET, int kt, int buf, int q) __attribute__((always_inline)) {
        constexpr int set = decltype(SET)::value;
        const int t = q >> 1;
        char* dst = smem + buf * (2 * TILE_BYTES) + wave * 1024 + t * 4096 + ((q & 1) ? TILE_BYTES : 0);
        if constexpr (SHARED) {
            // per-lane 64-bit addresses: this variant is short of scalar registers, and a buffer descriptor that the
            // register allocator moves into vector registers would be re-broadcast lane by lane at every load
            const char* src = reinterpret_cast<const char*>((q & 1) ? wbase : xbase) + ((q & 1) ? wo[t] : xo[t]) + kt * (BK * 2);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src, (lptr_t)dst, 16, 0, 0);
        } else {
            if (q & 1) __builtin_amdgcn_raw_ptr_buffer_load_lds(src_rsw[set], (lptr_t)dst, 16, src_vw[set] + t * src_gw[set], src_so[set], 0, 0);
            else __builtin_amdgcn_raw_ptr_buffer_load_lds(src_rsx[set], (lptr_t)dst, 16, src_vx[set] + t * src_gx[set], src_so[set], 0, 0);
        }
    };
    // One block = the 16 MFMAs of sub-step S_CUR in a fixed issue order (a scheduling barrier after every group keeps
    // the compiler from regrouping): even slots carry one fragment read each (for the next block), odd slots carry
    // the direct loads D0..D1-1 of slice lkt, spread evenly.
    auto block = [&](auto S_CUR, int rbuf, auto RKK, auto RS, auto SET, int lkt, int lbuf, auto D0, auto D1) __attribute__((always_inline)) {
        constexpr int s_cur = decltype(S_CUR)::value, rkk = decltype(RKK)::value, rs = decltype(RS)::value;
        constexpr int d0 = decltype(D0)::value, d1 = decltype(D1)::value, n = d1 - d0;
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            mfma1(s_cur, q);
            const int o = q >> 1;
            if (!(q & 1)) frag1(rbuf, rkk, rs, o);
            else if (((o + 1) * n) / 8 > (o * n) / 8) dma1(SET, lkt, lbuf, d0 + (o * n) / 8);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // the 16 direct loads of a slice ride on consecutive blocks: the last block of the slice before the previous one's
    // (N3), then the first blocks of the previous slice (N0, N1), none in the block before the wait.  As early as the
    // buffer allows: with the fused loss other tiles' target reads are in flight and operand loads take longer, and the
    // early split gains 2 % there (a later one, 6 / 6 / 4, was 0.7 % faster for a forward without a loss).
    constexpr int N3 = 8, N0 = 8, N1 = 0;
    static_assert(N3 + N0 + N1 == 16, "loads per slice");
    // plain slices kt0 .. kt1-1 of the steady state; on entry fragment set 0 holds sub-step 0 of slice kt0 and the
    // first N3 loads of slice kt0+1 are in flight; the same holds for kt1 on exit
    auto steady = [&](int kt0, int kt1) __attribute__((always_inline)) {
        for (int kt = kt0; kt < kt1; ++kt) {
            const int cur = kt & 1;
            select_slice(IC<0>{}, kt + 1);
            block(IC<0>{}, cur, IC<1>{}, IC<1>{}, IC<0>{}, kt + 1, cur ^ 1, IC<N3>{}, IC<N3 + N0>{});
            block(IC<1>{}, cur, IC<2>{}, IC<0>{}, IC<0>{}, kt + 1, cur ^ 1, IC<N3 + N0>{}, IC<16>{});
            block(IC<0>{}, cur, IC<3>{}, IC<1>{}, IC<0>{}, 0, 0, IC<0>{}, IC<0>{});
            // every operand load of the next slice has landed; all waves are done reading the buffer that the next
            // loads overwrite
            __builtin_amdgcn_s_waitcnt(0x0070);              // vmcnt(0) lgkmcnt(0)
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            // past the last pipelined slice the loads re-fetch it into the buffer nobody reads any more
            const int k2 = min(kt + 2, npipe - 1);
            select_slice(IC<1>{}, k2);
            block(IC<1>{}, cur ^ 1, IC<0>{}, IC<0>{}, IC<1>{}, k2, cur, IC<0>{}, IC<N3>{});
        }
    };
    // a slice whose operands are complete in buffer `buf`, fragment set 0 not yet read
    auto multiply_plain = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < 8; ++q) frag1(buf, 0, 0, q);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            if (kk + 1 < 4) {
#pragma unroll
                for (int q = 0; q < 8; ++q) frag1(buf, kk + 1, (kk + 1) & 1, q);
            }
#pragma unroll
            for (int q = 0; q < 16; ++q) mfma1(kk & 1, q);
        }
    };
    // the plain slices 0 .. nfull-1 (and ready-made extension slices) through the pipeline above
    auto run_plain = [&]() __attribute__((always_inline)) {
        if (npipe == 0) return;
        select_slice(IC<0>{}, 0);
#pragma unroll
        for (int q = 0; q < 16; ++q) dma1(IC<0>{}, 0, 0, q);
        if (npipe > 1) {
            select_slice(IC<1>{}, 1);
#pragma unroll
            for (int q = 0; q < N3; ++q) dma1(IC<1>{}, 1, 1, q);
            __builtin_amdgcn_s_waitcnt(0x0F70 | N3);      // vmcnt(N3): slice 0 has landed
        } else {
            __builtin_amdgcn_s_waitcnt(0x0F70);
        }
        __syncthreads();
        if (npipe > 1) {
#pragma unroll
            for (int q = 0; q < 8; ++q) frag1(0, 0, 0, q);
            steady(0, npipe - 1);
            __builtin_amdgcn_s_waitcnt(0x0F70);          // the re-fetches
            // last plain slice: sub-step 0 is already in fragment set 0
            const int cur = (npipe - 1) & 1;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                if (kk + 1 < 4) {
#pragma unroll
                    for (int q = 0; q < 8; ++q) frag1(cur, kk + 1, (kk + 1) & 1, q);
                }
#pragma unroll
                for (int q = 0; q < 16; ++q) mfma1(kk & 1, q);
            }
        } else {
            multiply_plain(0);
        }
        __syncthreads();
    };
    // slices [it_begin, it_end) that the threads fill themselves (ragged end of d_in, rank-r extension), one at a time
    auto run_manual = [&](int it_begin, int it_end) __attribute__((always_inline)) {
        for (int it = it_begin; it < it_end; ++it) {
            fill_manual(it, 0);
            __syncthreads();
            multiply_plain(0);
            __syncthreads();
        }
    };
    // ---- evaluation point: the accumulators hold Y0 (shared mode, after the d_in slices), or Y with
    // the rank-r term of the current sign.  Lane = one token, 16 consecutive outputs per block.
    // Differences and their squares are taken in fp32, four at a time, and summed in fp64.
    auto evaluate = [&](int phase) __attribute__((always_inline)) {
        double part = 0.0;
        // shared mode: the first evaluation turns the accumulators into the residual Y0 - Y*, so the
        // target is read once and the two perturbed evaluations are sums of squares of registers
        const bool resid = !CE && SHARED && phase > 0 && p.loss_kind == AGZO_LOSS_MSE;
        auto eval_block = [&](auto J) __attribute__((always_inline)) {
            constexpr int j = decltype(J)::value;
            const int64_t row = m0 + wb * (BT / WB) + j * 32 + lr;
#pragma clang loop unroll(full)
            for (int i = 0; i < BA; ++i) {
                const int64_t col0 = n0 + wa * (BT / WA) + i * 32 + lh * 16;
                floatx16 v = acc[i][j];
                if (row >= p.M || col0 >= p.N) continue;
                if (resid) {
#pragma clang loop unroll(full)
                    for (int q = 0; q < 4; ++q) {
                        float s4 = 0.f;
#pragma clang loop unroll(full)
                        for (int u = 0; u < 4; ++u)
                            if (col0 + 4 * q + u < p.N) s4 = fmaf(v[4 * q + u], v[4 * q + u], s4);
                        part += (double)s4;
                    }
                    continue;
                }
                if (p.vec_ok && col0 + 16 <= p.N) {
                    if (y_f32) {
                        float4* dst = reinterpret_cast<float4*>(reinterpret_cast<float*>(p.Y) + row * p.ldy + col0);
#pragma clang loop unroll(full)
                        for (int q = 0; q < 4; ++q) dst[q] = make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
                    }
                    if (y_bf16) {
                        uint4* dst = reinterpret_cast<uint4*>(reinterpret_cast<bf16_t*>(p.Y) + row * p.ldy + col0);
                        uint32_t w[8];
#pragma clang loop unroll(full)
                        for (int q = 0; q < 8; ++q) w[q] = pack_bf16x2(v[2 * q], v[2 * q + 1]);
                        dst[0] = make_uint4(w[0], w[1], w[2], w[3]);
                        dst[1] = make_uint4(w[4], w[5], w[6], w[7]);
                    }
                    if (l_f32) {
#pragma clang loop unroll(full)
                        for (int q = 0; q < 4; ++q) {
                            const uint4 t = reinterpret_cast<const uint4*>(reinterpret_cast<const float*>(p.target) + row * p.ldt + col0)[q];
                            const float tv[4] = {__uint_as_float(t.x), __uint_as_float(t.y), __uint_as_float(t.z), __uint_as_float(t.w)};
                            float s4 = 0.f;
#pragma clang loop unroll(full)
                            for (int u = 0; u < 4; ++u) {
                                const float dd = v[4 * q + u] - tv[u];
                                s4 = fmaf(dd, dd, s4);
                                if (SHARED) v[4 * q + u] = dd;
                            }
                            part += (double)s4;
                        }
                    }
                    if (l_bf16) {
#pragma clang loop unroll(full)
                        for (int q = 0; q < 2; ++q) {
                            const uint4 t = reinterpret_cast<const uint4*>(reinterpret_cast<const bf16_t*>(p.target) + row * p.ldt + col0)[q];
                            const uint32_t tw[4] = {t.x, t.y, t.z, t.w};
#pragma clang loop unroll(full)
                            for (int h = 0; h < 2; ++h) {
                                float s4 = 0.f;
#pragma clang loop unroll(full)
                                for (int u = 0; u < 2; ++u) {
                                    const uint32_t w = tw[2 * h + u];
                                    const float d0 = v[8 * q + 4 * h + 2 * u] - __uint_as_float(w << 16);
                                    const float d1 = v[8 * q + 4 * h + 2 * u + 1] - __uint_as_float(w & 0xFFFF0000u);
                                    s4 = fmaf(d0, d0, s4);
                                    s4 = fmaf(d1, d1, s4);
                                    if (SHARED) { v[8 * q + 4 * h + 2 * u] = d0; v[8 * q + 4 * h + 2 * u + 1] = d1; }
                                }
                                part += (double)s4;
                            }
                        }
                    }
                } else {
#pragma clang loop unroll(full)
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
                                if (SHARED) v[e] = dd;
                            }
                        }
                    }
                }
                if (SHARED) acc[i][j] = v;
            }
        };
        eval_block(IC<0>{});
        eval_block(IC<1>{});
        eval_block(IC<2>{});
        eval_block(IC<3>{});
        if (CE) {
            // a lane holds 16 of the 32 logits of each of its BA blocks for BB tokens; its partner lane
            // (lane ^ 32) holds the other 16.  Online softmax over the wave's columns, per token.
#pragma clang loop unroll(full)
            for (int j = 0; j < BB; ++j) {
                const int64_t row = m0 + wb * (BT / WB) + j * 32 + lr;
                const int tgt = (row < p.M) ? p.ce_target[row] : -1;
                float mx = -INFINITY, tl = 0.f;
                bool has_tl = false;
                // per block: how many of the lane's 16 columns exist, and which of them (if any) is the target
                int ncol[BA], trel[BA];
#pragma clang loop unroll(full)
                for (int i = 0; i < BA; ++i) {
                    const int64_t col0 = n0 + wa * (BT / WA) + i * 32 + lh * 16;
                    ncol[i] = (int)max((int64_t)0, min((int64_t)16, p.N - col0));
                    trel[i] = (tgt >= 0) ? (int)((int64_t)tgt - col0) : -1;
                }
#pragma clang loop unroll(full)
                for (int i = 0; i < BA; ++i) {
#pragma clang loop unroll(full)
                    for (int e = 0; e < 16; ++e) {
                        const float y = acc[i][j][e];
                        if (e < ncol[i]) mx = fmaxf(mx, y);
                        if (e == trel[i]) { tl = y; has_tl = true; }
                    }
                }
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                // exp(y - mx) as 2^((y - mx) log2 e) on the hardware exponential: the difference is exact enough in
                // fp32 (one rounding), the terms that matter have small exponents, and the far tail underflows to 0
                float sm = 0.f;
#pragma clang loop unroll(full)
                for (int i = 0; i < BA; ++i) {
#pragma clang loop unroll(full)
                    for (int e = 0; e < 16; ++e)
                        if (e < ncol[i]) sm += __builtin_amdgcn_exp2f((acc[i][j][e] - mx) * 1.44269504088896341f);
                }
                sm += __shfl_xor(sm, 32);
                if (row < p.M) {
                    const int64_t chunk = tn * WA + wa;
                    const int64_t nchunk = (int64_t)p.tiles_n * WA;
                    if (lh == 0) p.ce_ms[((int64_t)phase * nchunk + chunk) * p.M + row] = make_float2(mx, sm);
                    if (has_tl) p.ce_tl[(int64_t)phase * p.M + row] = tl;
                }
            }
        }
        if (!CE && p.loss_kind == AGZO_LOSS_MSE) {
            red[tid] = part;
            __syncthreads();
            for (int s = NT / 2; s > 0; s >>= 1) {
                if (tid < s) red[tid] += red[tid + s];
                __syncthreads();
            }
            if (tid == 0) p.partials[(int64_t)phase * p.tiles_m * p.tiles_n + tm * p.tiles_n + tn] = red[0];
            __syncthreads();
        }
    };
    if (SHARED && next > 0) {
        run_plain();
        // one copy of the fill / multiply / evaluate code, walked three times: Y0, Y+ (extension with +eps), Y- (-2 eps)
        for (int ph = 0; ph < 3; ++ph) {
            const int it0 = (ph == 0) ? nfull : nd + (ph - 1) * next;
            const int it1 = nd + ph * next;
            run_manual(it0, it1);
            evaluate(ph);
        }
    } else if (ext_dma) {
        // pipelined: plain slices, then the ready-made extension slices; the ragged end of d_in (if any) last
        run_plain();
        run_manual(nfull, nd);
        evaluate(0);
    } else {
        run_plain();
        run_manual(nfull, total);
        evaluate(0);
    }
    if (p.clk && blockIdx.x == 0 && tid == 0) { p.clk[2] = __builtin_readcyclecounter(); p.clk[3] = wall_clock64(); }
}



// Extension operands for one perturbed forward, written once instead of once per tile: eight columns per thread.
// Rows 0..M-1 are the X side ([Ph | Ph | Pl | 0], P = X B split hi + lo in bf16), rows M..M+N-1 the W side
// ([Gh | Gl | Gh | 0], G regenerated from the Philox seed, times the signed eps); n_w = 2 adds rows M+N..M+2N-1, the
// W side once more with coef2 (the shared-forward kernel's second pass, -2 eps).
__global__ __launch_bounds__(256) void gemm_ext_prep_kernel(bf16_t* __restrict__ Xext, bf16_t* __restrict__ Wext, int64_t M,
                                                            int64_t N, int ext_ld, const float* __restrict__ P, int r, int rp,
                                                            float coef, float coef2, int n_w, uint32_t s_lo, uint32_t s_hi) {
    const int chunks = ext_ld / 8;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (M + n_w * N) * chunks) return;
    int64_t row = idx / chunks;
    const bool second = row >= M + N;
    if (second) { row -= N; coef = coef2; }
    const int col0 = (int)(idx % chunks) * 8;
    const int seg = col0 / rp, k0 = col0 % rp;
    uint32_t hi[4] = {0, 0, 0, 0}, lo[4] = {0, 0, 0, 0};
    if (seg < 3) {
        float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (row < M) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (k0 + i < r) v[i] = P[row * r + k0 + i];
        } else {
            const int64_t j = row - M;
            if (k0 < r) {
                const float4 z = philox_normal4(s_lo, s_hi, AGZO_TAG_G, (uint32_t)j, (uint32_t)(k0 >> 2));
                v[0] = z.x; v[1] = z.y; v[2] = z.z; v[3] = z.w;
            }
            if (k0 + 4 < r) {
                const float4 z = philox_normal4(s_lo, s_hi, AGZO_TAG_G, (uint32_t)j, (uint32_t)((k0 >> 2) + 1));
                v[4] = z.x; v[5] = z.y; v[6] = z.z; v[7] = z.w;
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = (k0 + i < r) ? coef * v[i] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            hi[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
            lo[i] = pack_bf16x2(v[2 * i] - __uint_as_float(hi[i] << 16), v[2 * i + 1] - __uint_as_float(hi[i] & 0xFFFF0000u));
        }
    }
    // X side: [hi | hi | lo]; W side: [hi | lo | hi]
    const bool use_lo = (row < M) ? (seg == 2) : (seg == 1);
    const uint4 out = use_lo ? make_uint4(lo[0], lo[1], lo[2], lo[3]) : make_uint4(hi[0], hi[1], hi[2], hi[3]);
    bf16_t* dst = (row < M) ? Xext + row * ext_ld + col0 : Wext + (row - M + (second ? N : 0)) * ext_ld + col0;
    *reinterpret_cast<uint4*>(dst) = out;
}

size_t gemm_bf16_ext_bytes(int64_t M, int64_t N, int r) {
    const int rp = (r + 15) / 16 * 16;
    const int ext_ld = (3 * rp + BK - 1) / BK * BK;
    return (size_t)(M + 2 * N) * ext_ld * sizeof(bf16_t);   // X side, W side, and the W side of a second pass
}

template <int WA, int WB, bool SHARED, int EPI>
static hipError_t launch_variant(const GemmParams& p, hipStream_t st) {
    static bool attr_set = false;
    const int smem = 4 * TILE_BYTES + 64 * WA * WB * (int)sizeof(double);
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_bf16_kernel<WA, WB, SHARED, EPI>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid((unsigned)((int64_t)p.tiles_m * p.tiles_n));
    hipLaunchKernelGGL((gemm_bf16_kernel<WA, WB, SHARED, EPI>), grid, dim3(64 * WA * WB), smem, st, p);
    return hipGetLastError();
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
    p.tiles_m = (int)((a.M + BT - 1) / BT);
    p.tiles_n = (int)((a.N + BT - 1) / BT);
    // a band of group_m token tiles per XCD run stays hot while the output tiles sweep past; a deep d_in makes the
    // band too large for the last-level cache, so it is halved there (measured on the 12288-wide down projection)
    p.group_m = (a.K >= 8192) ? 4 : 8;
    bool vec = true;
    if (a.Y) vec = vec && (a.ldy % 8 == 0) && ((reinterpret_cast<uintptr_t>(a.Y) & 15) == 0);
    if (a.loss.kind == AGZO_LOSS_MSE)
        vec = vec && (a.loss.ldt % 8 == 0) && ((reinterpret_cast<uintptr_t>(a.loss.target) & 15) == 0);
    p.vec_ok = vec ? 1 : 0;
    p.shared = a.shared ? 1 : 0;
    p.Xext = nullptr; p.Wext = nullptr; p.Wext2 = nullptr; p.ext_ld = 0;
    const bool small = small_shape(a.M, a.N) && !a.large_tiles && !a.shared && p.loss_kind != AGZO_LOSS_CE;
    // the kernel of gemm_bf16_aligned.hip takes tile-aligned layers: squared error without a stored Y (also in
    // shared-forward mode), the cross-entropy statistics without a stored Y, or a stored bf16 Y without a loss
    const bool aligned_shape = !small && vec && a.M % BT == 0 && a.N % BT == 0 && a.K % BK == 0 && a.K >= 2 * BK && (!a.P || a.ext_ws);
    const bool mse = aligned_shape && ((a.loss.kind == AGZO_LOSS_MSE && !a.Y) ||
                                       (a.loss.kind == AGZO_LOSS_CE && !a.Y && !a.shared) ||
                                       (a.loss.kind == AGZO_LOSS_NONE && a.Y && a.y_dtype == AGZO_BF16 && !a.shared));
    if (a.P && a.ext_ws && (!a.shared || mse)) {
        p.ext_ld = (3 * p.rp + BK - 1) / BK * BK;
        bf16_t* xe = static_cast<bf16_t*>(a.ext_ws);
        bf16_t* we = xe + a.M * p.ext_ld;
        const int n_w = a.shared ? 2 : 1;
        const int64_t items = (a.M + n_w * a.N) * (p.ext_ld / 8);
        hipLaunchKernelGGL(gemm_ext_prep_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, st, xe, we, a.M, a.N, p.ext_ld,
                           a.P, a.r, p.rp, a.eps_signed, -2.f * a.eps_signed, n_w, p.s_lo, p.s_hi);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        p.Xext = xe; p.Wext = we;
        if (a.shared) p.Wext2 = we + a.N * p.ext_ld;
    }
    p.ce_target = reinterpret_cast<const int32_t*>(a.loss.target);
    p.ce_ms = reinterpret_cast<float2*>(a.loss.ce_ms);
    p.ce_tl = a.loss.ce_tl;
    p.clk = a.clk;
    p.sk_T = nullptr; p.sk_mpad = 0; p.sk_partial = nullptr;
    if (a.sk_T) {
        if (!small || a.P || !gemm_bf16_fuses_sketch(a.M, a.N, a.r, a.large_tiles)) return hipErrorInvalidValue;
        p.sk_T = a.sk_T; p.sk_mpad = a.sk_mpad; p.sk_partial = a.sk_partial;
    }
    if (small) {
        // the workspace was sized for this tiling's partials (gemm_bf16_num_workgroups with small_ok)
        if (a.P && !p.Xext) return hipErrorInvalidValue;      // the small tiling takes the rank-r term as operands only
        p.tiles_m = (int)((a.M + BT_SMALL - 1) / BT_SMALL);
        p.tiles_n = (int)((a.N + BT_SMALL - 1) / BT_SMALL);
        return launch_gemm_bf16_small(p, st);
    }
    if (mse) return launch_gemm_bf16_aligned(p, st);
    const bool ce = p.loss_kind == AGZO_LOSS_CE;
    if (p.shared) return ce ? launch_variant<2, 2, true, 1>(p, st) : launch_variant<2, 2, true, 0>(p, st);
    return ce ? launch_variant<2, 2, false, 1>(p, st) : launch_variant<2, 2, false, 0>(p, st);
}

}  // namespace agzo
