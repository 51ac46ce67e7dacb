// Forward GEMM for tile-aligned layers, the case the benchmark configurations run:
//     OUT = 0:  f = sum over the tile of (X W^T (+ eps (X B) G^T) - Y*)^2     (f0, f+, f- of Sec. 4.1; Eq. 7 factored)
//     OUT = 1:  Y = X W^T (+ eps (X B) G^T) stored as bf16                     (a layer inside a model, Alg. 2)
//     OUT = 2:  the same logits never stored: per token and 128-column chunk their maximum and the sum of exponentials
//               around it, and the target's logit (token cross-entropy of a model's last layer; loss.hip combines them)
// Same tile, tile layout in LDS and direct global -> LDS operand loads as gemm_bf16.hip (256 x 256 tile, four waves of
// 128 x 128, 64-wide K slices), but a kernel of its own with one straight path and nothing else compiled in: M and N
// multiples of 256, d_in a multiple of 64 and at least 128, 16-byte aligned target / output rows, the rank-r extension
// as prepared operands.
//
// Matrix instruction.
// v_mfma_f32_16x16x32_bf16, 8 x 8 blocks per wave, two k steps of 32 per slice, where gemm_bf16.hip has 4 x 4 blocks of
// v_mfma_f32_32x32x16_bf16 and four k steps.  Both give the published rate at the top clock; under the device's power
// limit, on random operands, a register-only loop of the first holds 2.2 PFLOP/s at 2.1 GHz and one of the second
// 1.9 at 1.8, and this kernel spends 80 - 90 % of its time in these instructions.  A slice is four blocks of 32
// instructions (block rows 0..3 / 4..7 of k step 0, then of k step 1), each walked token block by token block with the
// four W fragments of its block rows and the eight X fragments of the k step in registers; the W fragments of the next
// block are read in the first half of a block, and in the second block of a k step each X fragment is replaced by the
// next k step's as soon as its last instruction has issued.
//
// LDS stages.
// A 64-wide slice is 32 KiB per operand and the compute unit has 160 KiB: three stages for W and two for X.  A stage
// can be filled again once every wave has read its last fragment, which the one barrier of a slice establishes (after
// the third of its four blocks of matrix instructions: fragments are read a block ahead).  With two stages per
// operand everything for the slice after next had to be requested behind that barrier and to land before the next
// one, the later half of it within two blocks: the barrier waited for the slowest line, 250 - 450 cycles per slice on
// the wide layers.  With the third W stage the W half of the slice after next is requested a block before the barrier,
// into the stage the previous slice left, and has six blocks to land; behind the barrier only the X half is
// requested, at once, and has three.  The wait in front of the barrier is for all but the eight youngest loads (loads
// return in the order issued).  Cycles per launch fell by 15 % on the wide layers; the clock, which the power limit
// sets, gave a third of that back.
//
// Squared error (OUT = 0).
// The accumulators do not start at zero but at minus the target tile: the target is requested before the first
// operand slice and converted while that slice is on its way, so after the last slice the registers hold the residual
// Y - Y* and the epilogue is a sum of squares of registers with no memory access.  (Reading the target in the epilogue
// left the matrix cores idle for 15 - 18 % of a tile: every workgroup asks for its 128 KiB at the same moment and
// waits out the latency, and the staging registers spilled.)  All evaluations of a step start from the same -Y*, so
// f+ and f- still share bit-identical accumulators up to the rank-r slices.
//
// Persistent workgroups.
// One workgroup per compute unit walks through a list of tiles (its LDS and accumulators leave no room for a second one,
// so a workgroup per tile paid the launch of a workgroup, the latency of the first operand slices and of the target, and
// an unpipelined last slice once per tile, with the matrix cores idle; walking tile lists instead measured 1 - 3 % faster).  The slice
// loop runs across tile boundaries: every slice, the last one of a tile included, is a steady iteration whose loads
// fetch the slice after next - at the end of a tile the first two slices of the next tile - so when a tile's last
// matrix instruction has issued, the next tile's first slice is in LDS and its first fragments are in registers.
// Between two tiles only the accumulators change hands: the next target is requested, the finished tile is evaluated
// (or stored) while it travels, and the accumulators restart from minus the new target.  The tile list keeps the
// order that makes an XCD's 32 workgroups share operand slices in its L2: XCD x (workgroup id mod 8) owns a contiguous
// run of tiles, and its workgroups take them 32 at a time.
//
// PHASES = 3 is the shared-forward schedule for a single layer: the d_in slices are multiplied once, f0 is the sum of
// squares of the accumulators as they stand, the extension slices with +eps make them the residual of f+, the same
// slices with -2 eps that of f-.  The extension operands of both passes are requested before the evaluation that
// precedes them, so their latency runs under it.
#include "gemm_bf16_common.h"

namespace agzo {

typedef float floatx4 __attribute__((ext_vector_type(4)));

// LDS row m' of a 64-row group of the W tile holds W row perm64(m'): block t = m' / 16 of the group, output register e
// of lane group g = (m' / 4) mod 4 of a 16 x 16 block is row 4 g + e of the block, which this makes output column
// 16 g + 4 t + e of the group: a lane's 4 x 4 values over four neighbouring blocks are 16 consecutive outputs.
__device__ __forceinline__ int w_perm64(int m) { return ((m >> 2) & 3) * 16 + (m >> 4) * 4 + (m & 3); }

// buffer descriptor over everything from `base` on (no range check: the kernel only takes tiles that lie inside)
__device__ __forceinline__ __amdgpu_buffer_rsrc_t rsrc(const bf16_t* base) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(base), 0, (int)0xFFFFFFFFu, 0x00020000);
}

// A value moved into an accumulation register by hand: the 256 start values of the accumulators are produced by
// vector instructions, and left to itself the compiler parks them in ordinary registers (and spills most of them)
// until the first multiply.
__device__ __forceinline__ float to_acc(float x) {
    float r;
    asm volatile("v_accvgpr_write_b32 %0, %1" : "=a"(r) : "v"(x));
    return r;
}

// ... and read back by hand, one value at a time in program order: left to itself the compiler copies all 256
// accumulators into ordinary registers at once before it sums their squares, and whatever else is live at that moment
// (the next tile's target) goes to scratch memory.  The compiler's hazard bookkeeping does not look inside the asm:
// the caller keeps the wait states that a matrix instruction needs before its result may be read (19 for the longest).
__device__ __forceinline__ float from_acc(float x) {
    float r;
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(r) : "a"(x));
    return r;
}

template <int OUT, bool T_F32, int PHASES>
__global__ __launch_bounds__(256) void gemm_bf16_aligned_kernel(GemmParams p) {
    static_assert(OUT == 0 || (PHASES == 1 && !T_F32), "the kernels without a squared-error target have one evaluation");
    constexpr int NT = 256, BA = 4, BB = 4;
    constexpr int W_BASE = 0, X_BASE = 3 * TILE_BYTES;       // LDS: three W stages, then two X stages (all 160 KiB)
    extern __shared__ __align__(16) char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    if (p.clk && blockIdx.x == 0 && tid == 0) { p.clk[0] = __builtin_readcyclecounter(); p.clk[1] = wall_clock64(); }
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wa = wave >> 1, wb = wave & 1;
    const int lc = lane & 15, lg = lane >> 4;      // matrix instruction 16x16x32: column (token) / row of a fragment, k group

    // ---- this workgroup's tiles ---------------------------------------------------------------------
    // XCD x = id mod 8 (ids are dealt round-robin over the XCDs) owns the run of tiles [x per, (x + 1) per), walked by
    // its S workgroups S at a time; the up to 7 tiles left over go to the last workgroup of the first XCDs.  Inside a
    // run, tiles are ordered in bands of group_m token tiles per output tile, so that the tiles an XCD works on at any
    // moment share a few W tiles and a band of X tiles.
    const int nwg = p.tiles_m * p.tiles_n;
    const int G = (int)gridDim.x;
    const bool by_xcd = (G % 8 == 0);
    const int S = by_xcd ? G / 8 : G;
    const int xcd = by_xcd ? (int)blockIdx.x % 8 : 0, slot = by_xcd ? (int)blockIdx.x / 8 : (int)blockIdx.x;
    const int per = by_xcd ? nwg / 8 : nwg;
    const int n_run = slot < per ? (per - slot + S - 1) / S : 0;
    const int n_tiles = __builtin_amdgcn_readfirstlane(n_run + ((by_xcd && slot == S - 1 && xcd < nwg - 8 * per) ? 1 : 0));
    const int GROUP_M = p.group_m;
    int64_t tm = 0, tn = 0;
    auto tile_at = [&](int i, int64_t& tm_, int64_t& tn_) __attribute__((always_inline)) {
        const int lin = (i < n_run) ? xcd * per + slot + i * S : 8 * per + xcd;
        const int group = lin / (GROUP_M * p.tiles_n);
        const int first_m = group * GROUP_M;
        const int gsz = min(GROUP_M, p.tiles_m - first_m);
        const int in_group = lin - group * GROUP_M * p.tiles_n;
        tm_ = __builtin_amdgcn_readfirstlane(first_m + in_group % gsz);
        tn_ = __builtin_amdgcn_readfirstlane(in_group / gsz);
    };
    if (n_tiles == 0) return;
    tile_at(0, tm, tn);
    int64_t m0 = tm * BT, n0 = tn * BT;

    // ---- operand sources: X / W slices, then the prepared extension operands ----------------------
    const bool has_ext = p.Xext != nullptr;
    // operand bases of the current tile (d_in slices, extension slices) and of the next tile's d_in slices
    const bf16_t *xb, *wb_, *xb2, *wb2, *wb3, *xbn, *wbn;
    auto tile_sources = [&]() __attribute__((always_inline)) {
        xb = p.X + m0 * p.ldx;
        wb_ = p.W + n0 * p.ldw;
        xb2 = has_ext ? p.Xext + m0 * p.ext_ld : xb;
        wb2 = has_ext ? p.Wext + n0 * p.ext_ld : wb_;
        wb3 = (has_ext && PHASES == 3) ? p.Wext2 + n0 * p.ext_ld : wb_;
    };
    // i: index of the tile after the current one; past the list: the current tile once more (its first slices are
    // fetched again into the stage nobody reads)
    auto next_sources = [&](int i) __attribute__((always_inline)) {
        int64_t tmn = tm, tnn = tn;
        if (i < n_tiles) tile_at(i, tmn, tnn);
        xbn = p.X + tmn * BT * p.ldx;
        wbn = p.W + tnn * BT * p.ldw;
    };
    tile_sources();
    next_sources(1);
    // LDS row 32 t + row0 of a tile: X row 32 t + row0; W row 64 (t / 2) + 8 (t mod 2) + perm64(row0) (perm64 of a row 32
    // further on is 8 more)
    const int row0 = 8 * wave + (lane >> 3);
    const int chunk0 = (lane & 7) ^ ((row0 >> 1) & 7);       // the swizzle term does not depend on t
    const int vx = (int)(((int64_t)row0 * p.ldx + chunk0 * 8) * 2), vw = (int)(((int64_t)w_perm64(row0) * p.ldw + chunk0 * 8) * 2);
    const int vx2 = (row0 * p.ext_ld + chunk0 * 8) * 2, vw2 = (w_perm64(row0) * p.ext_ld + chunk0 * 8) * 2;
    const int gsx = (int)(64 * p.ldx), gsw = (int)(64 * p.ldw), gs2 = 64 * p.ext_ld;   // bytes between row groups
    const int nfull = (int)(p.K / BK);
    const int next = has_ext ? p.ext_ld / BK : 0;
    // slices that ride the load pipeline: the d_in slices, and in the one-evaluation kernel the extension behind them
    // (at least two: the first two slices of a tile are always d_in slices)
    const int npipe = nfull + (PHASES == 1 ? next : 0);
    typedef __attribute__((address_space(3))) void* lptr_t;

    // ---- accumulators <- minus the target tile ----------------------------------------------------
    // 8 x 8 blocks of 16 x 16 per wave.  Lane (lc, lg) holds token 16 J + lc of token block J and, over the four output
    // blocks 4 I4 .. 4 I4 + 3, the 16 consecutive outputs 64 I4 + 16 lg + [0, 16): value 4 t + e is register e of block
    // 4 I4 + t.  The raw 16-byte vectors of the target wait in 128 registers that nothing else needs before the first
    // multiply: a whole bf16 tile, or half an fp32 one (token blocks 0..3, then 4..7)
    floatx4 acc[8][8];
    uint4 traw[32];
    auto tload = [&](auto JJ) __attribute__((always_inline)) {
        constexpr int J = decltype(JJ)::value;
        const int64_t row = m0 + wb * 128 + J * 16 + lc;
        const int64_t colw = n0 + wa * 128 + lg * 16;
        if (T_F32) {
            const uint4* src = reinterpret_cast<const uint4*>(reinterpret_cast<const float*>(p.target) + row * p.ldt + colw);
#pragma clang loop unroll(full)
            for (int i4 = 0; i4 < 2; ++i4)
#pragma clang loop unroll(full)
                for (int q = 0; q < 4; ++q) traw[(J & 3) * 8 + i4 * 4 + q] = src[i4 * 16 + q];
        } else {
            const uint4* src = reinterpret_cast<const uint4*>(reinterpret_cast<const bf16_t*>(p.target) + row * p.ldt + colw);
#pragma clang loop unroll(full)
            for (int i4 = 0; i4 < 2; ++i4)
#pragma clang loop unroll(full)
                for (int q = 0; q < 2; ++q) traw[J * 4 + i4 * 2 + q] = src[i4 * 8 + q];
        }
    };
    auto tneg = [&](auto JJ) __attribute__((always_inline)) {
        constexpr int J = decltype(JJ)::value;
#pragma clang loop unroll(full)
        for (int i4 = 0; i4 < 2; ++i4) {
            float v[16];
            if (T_F32) {
#pragma clang loop unroll(full)
                for (int q = 0; q < 4; ++q) {
                    const uint4 t = traw[(J & 3) * 8 + i4 * 4 + q];
                    v[4 * q] = -__uint_as_float(t.x); v[4 * q + 1] = -__uint_as_float(t.y);
                    v[4 * q + 2] = -__uint_as_float(t.z); v[4 * q + 3] = -__uint_as_float(t.w);
                }
            } else {
#pragma clang loop unroll(full)
                for (int q = 0; q < 2; ++q) {
                    const uint4 t = traw[J * 4 + i4 * 2 + q];
                    const uint32_t w[4] = {t.x, t.y, t.z, t.w};
#pragma clang loop unroll(full)
                    for (int u = 0; u < 4; ++u) {     // widened to fp32 with the sign flipped on the raw bits (one
                        // instruction each: adding 2^31 to the shifted word flips its top bit)
                        v[8 * q + 2 * u] = __uint_as_float((w[u] << 16) + 0x80000000u);
                        v[8 * q + 2 * u + 1] = __uint_as_float((w[u] & 0xFFFF0000u) ^ 0x80000000u);
                    }
                }
            }
#pragma clang loop unroll(full)
            for (int t = 0; t < 4; ++t) {
                floatx4 o;
#pragma clang loop unroll(full)
                for (int e = 0; e < 4; ++e) o[e] = to_acc(v[4 * t + e]);
                acc[i4 * 4 + t][J] = o;
            }
        }
    };

    // ---- multiply ---------------------------------------------------------------------------------
    // v_mfma_f32_16x16x32_bf16: two k steps of 32 per slice.  Fragment of block row I (W) or token block J (X), k step s:
    // lane (lc, lg) reads 16-byte chunk 4 s + lg of tile row 16 I + lc.  (The same flop count from this instruction
    // draws less power than from the 32x32x16 one: under the device's power limit the register-only probe holds
    // 2.2 PFLOP/s with it against 1.9.)
    int aoff[2], boff[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        aoff[ks] = W_BASE + lds_off(wa * 128 + lc, ks * 4 + lg);
        boff[ks] = X_BASE + lds_off(wb * 128 + lc, ks * 4 + lg);
    }
    bf16x8 aw[2][4], bx[8];                      // W fragments of four block rows, two sets; X fragments of the eight token blocks
    auto read_w = [&](int wbuf, int ks, int set, int i) __attribute__((always_inline)) {      // block row 4 set + i
        aw[set][i] = *reinterpret_cast<const bf16x8*>(smem + wbuf * TILE_BYTES + aoff[ks] + (set * 4 + i) * 2048);
    };
    auto read_x = [&](int xbuf, int ks, int J) __attribute__((always_inline)) {
        bx[J] = *reinterpret_cast<const bf16x8*>(smem + xbuf * TILE_BYTES + boff[ks] + J * 2048);
    };
    auto mfma1 = [&](int set, int i, int J) __attribute__((always_inline)) {
        // (written out, with the accumulator tied to one register tuple: through the builtin the compiler rotated a dozen
        // tuples per slice through vector registers)
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[set * 4 + i][J]) : "v"(aw[set][i]), "v"(bx[J]));
    };
    // source of a pipelined slice, chosen once per slice with scalar selects (no branches at the load sites)
    __amdgpu_buffer_rsrc_t src_rsx = rsrc(xb), src_rsw = rsrc(wb_);
    int src_so = 0;
    // vector offsets of a lane's eight row groups per operand, kept in registers: worked out in front of each load they
    // put an add and its latency between a matrix instruction and the load behind it
    int src_vxt[8], src_vwt[8];
    auto set_offsets = [&](int v0x, int gx, int v0w, int gw) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < 8; ++t) { src_vxt[t] = v0x + t * gx; src_vwt[t] = v0w + (t >> 1) * (2 * gw) + (t & 1) * (gw >> 2); }
    };
    set_offsets(vx, gsx, vw, gsw);
    // kt counts from the current tile's first slice; npipe and npipe + 1 are the first two slices of the next tile.
    // Two rounds of selects, each on one condition, between values (a select between captured references becomes a
    // computed address into the closure, which then stays in memory with everything it points to; and selects on
    // mixed conditions cost four scalar instructions each instead of one)
    auto select_slice = [&](int kt) __attribute__((always_inline)) {
        // (copies first: the selects then see values, not addresses of captured variables)
        const bf16_t *cxb = xb, *cwb = wb_, *cxb2 = xb2, *cwb2 = wb2, *cxbn = xbn, *cwbn = wbn;
        const int cvx = vx, cvw = vw, cvx2 = vx2, cvw2 = vw2, cgsx = gsx, cgsw = gsw, cgs2 = gs2;
        const bool e = kt >= nfull;                          // extension operands (or, past npipe, the next tile)
        const bf16_t* xs = e ? cxb2 : cxb;
        const bf16_t* ws = e ? cwb2 : cwb;
        int svx = e ? cvx2 : cvx, svw = e ? cvw2 : cvw, sgx = e ? cgs2 : cgsx, sgw = e ? cgs2 : cgsw;
        int so = e ? kt - nfull : kt;
        const bool nxt = kt >= npipe;
        xs = nxt ? cxbn : xs;
        ws = nxt ? cwbn : ws;
        svx = nxt ? cvx : svx;   svw = nxt ? cvw : svw;   sgx = nxt ? cgsx : sgx;   sgw = nxt ? cgsw : sgw;
        so = nxt ? kt - npipe : so;
        src_rsx = rsrc(xs);   src_rsw = rsrc(ws);
        set_offsets(svx, sgx, svw, sgw);
        src_so = so * (BK * 2);
    };
    // direct load of row group t (0..7) of the selected slice: X into X stage buf (0..1), W into W stage buf (0..2)
    auto dma_x = [&](int buf, int t) __attribute__((always_inline)) {
        char* dst = smem + X_BASE + buf * TILE_BYTES + wave * 1024 + t * 4096;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(src_rsx, (lptr_t)dst, 16, src_vxt[t], src_so, 0, 0);
    };
    auto dma_w = [&](int buf, int t) __attribute__((always_inline)) {
        char* dst = smem + W_BASE + buf * TILE_BYTES + wave * 1024 + t * 4096;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(src_rsw, (lptr_t)dst, 16, src_vwt[t], src_so, 0, 0);
    };
    // 32 MFMAs in fixed issue order: the block rows 4 SET .. 4 SET + 3 against the eight token blocks, token block by token
    // block, with the fragments in registers.  Rides along: the W fragments of the other set for the block after this one
    // (k step RKS of W stage rwbuf), one after the third instruction of every other token block; with REFILL, the X fragment
    // of token block J for the next k step (RKS of X stage rxbuf) as soon as the block's last instruction on it has issued;
    // the eight direct loads of one operand of the selected slice, one behind the first instruction of each token block
    // (LOADS: 0 none, 1 W, 2 X)
    auto block = [&](auto SET, auto RKS, auto REFILL, int rxbuf, int rwbuf, auto LOADS, int lbuf) __attribute__((always_inline)) {
        constexpr int set = decltype(SET)::value, rks = decltype(RKS)::value, loads = decltype(LOADS)::value;
        constexpr bool refill = decltype(REFILL)::value != 0;
#pragma unroll
        for (int J = 0; J < 8; ++J) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                mfma1(set, i, J);
                if (i == 0 && loads == 1) dma_w(lbuf, J);
                if (i == 0 && loads == 2) dma_x(lbuf, J);
                if (i == 2 && J < 4) read_w(rwbuf, rks, set ^ 1, J);
                if (i == 3 && refill) read_x(rxbuf, rks, J);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    // a slice whose operands are complete in buffer `buf`, unpipelined
    auto multiply_slice = [&](int buf, bool) __attribute__((always_inline)) {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
            for (int J = 0; J < 8; ++J) read_x(buf, ks, J);
#pragma unroll
            for (int set = 0; set < 2; ++set) {
#pragma unroll
                for (int i = 0; i < 4; ++i) read_w(buf, ks, set, i);
#pragma unroll
                for (int J = 0; J < 8; ++J)
#pragma unroll
                    for (int i = 0; i < 4; ++i) mfma1(set, i, J);
            }
        }
    };

    // ---- sum of squares of the accumulators    // ---- sum of squares of the accumulators: fp32 squares four at a time, summed in fp64; lanes, then waves, in a
    // fixed order ----
    // The four waves' sums meet in LDS, in `red`: the head of a W stage that nothing reads or fills at that moment
    // (the operand stages take all of the LDS)
    auto eval_sum = [&]() __attribute__((always_inline)) {
        double part = 0.0;
        // 24 wait states between the last matrix instruction and the first read of a result: the matrix instructions are
        // written out, so the compiler does not know of them and keeps no distance itself
        asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7");
#pragma clang loop unroll(full)
        for (int J = 0; J < 8; ++J)
#pragma clang loop unroll(full)
            for (int I = 0; I < 8; ++I) {
                const floatx4 v = acc[I][J];
                float s4 = 0.f;
#pragma clang loop unroll(full)
                for (int u = 0; u < 4; ++u) {
                    // (the shared-forward schedule multiplies on after an evaluation and nothing else is live there)
                    const float x = (PHASES == 1) ? from_acc(v[u]) : v[u];
                    s4 = fmaf(x, x, s4);
                }
                part += (double)s4;
            }
        return part;
    };
    auto eval_finish = [&](double part, int phase, int64_t tm_, int64_t tn_, double* red) __attribute__((always_inline)) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off);
        if (lane == 0) red[phase * 4 + wave] = part;
        __syncthreads();
        if (tid == 0)
            p.partials[(int64_t)phase * p.tiles_m * p.tiles_n + tm_ * p.tiles_n + tn_] =
                (red[phase * 4] + red[phase * 4 + 1]) + (red[phase * 4 + 2] + red[phase * 4 + 3]);
        // (one-evaluation kernel: the next slice's loads go into this stage, and no wave may issue them before the sums
        // have been read)
        if constexpr (PHASES == 1) __syncthreads();
    };
    auto evaluate = [&](int phase, int64_t tm_, int64_t tn_, double* red) __attribute__((always_inline)) {
        eval_finish(eval_sum(), phase, tm_, tn_, red);
    };

    // accumulators <- minus the target tile (squared error) or zero (stored output)
    auto start_tile = [&]() __attribute__((always_inline)) {
        if constexpr (OUT == 0) {
            tneg(IC<0>{}); tneg(IC<1>{}); tneg(IC<2>{}); tneg(IC<3>{});
            if (T_F32) { tload(IC<4>{}); tload(IC<5>{}); tload(IC<6>{}); tload(IC<7>{}); }
            tneg(IC<4>{}); tneg(IC<5>{}); tneg(IC<6>{}); tneg(IC<7>{});
        } else {
#pragma unroll
            for (int I = 0; I < 8; ++I)
#pragma unroll
                for (int J = 0; J < 8; ++J)
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[I][J][e] = 0.f;
        }
    };
    auto request_target = [&]() __attribute__((always_inline)) {
        if constexpr (OUT == 0) {
            tload(IC<0>{}); tload(IC<1>{}); tload(IC<2>{}); tload(IC<3>{});
            if (!T_F32) { tload(IC<4>{}); tload(IC<5>{}); tload(IC<6>{}); tload(IC<7>{}); }
        }
    };

    // ---- first tile: target and the first two slices ------------------------------------------------
    request_target();
    select_slice(0);
#pragma unroll
    for (int t = 0; t < 8; ++t) { dma_x(0, t); dma_w(0, t); }
    select_slice(1);
#pragma unroll
    for (int t = 0; t < 8; ++t) { dma_x(1, t); dma_w(1, t); }

    int g = 0;                                   // slices multiplied so far: slice g sits in W stage g mod 3, X stage g & 1
    int wst = 0;                                  // g mod 3
    for (int it = 0;; ++it) {
        // the accumulators are written here and nowhere else, and are dead at the end of the loop body: carried around
        // the loop they would pass through a join, which the compiler answers by spilling them
        start_tile();
        if (it == 0) {
            __builtin_amdgcn_s_waitcnt(0x4F70);              // vmcnt(16): slice 0 has landed
            __syncthreads();
#pragma unroll
            for (int J = 0; J < 8; ++J) read_x(0, 0, J);
#pragma unroll
            for (int i = 0; i < 4; ++i) read_w(0, 0, 0, i);
        }
        // every slice of the tile, the last one included, with its W in stage wst and its X in stage cur: on entry the X
        // fragments and W fragment set 0 hold its first k step, the next slice's W has landed or is in flight and its X is
        // in flight; the same holds for the next slice on exit
        for (int kt = 0; kt < npipe; ++kt, ++g) {
            const int cur = g & 1;
            const int wst1 = (wst == 2) ? 0 : wst + 1, wst2 = (wst == 0) ? 2 : wst - 1;      // stages of slices g + 1, g + 2
            // while the slice after next is a d_in slice of this tile only the K offset moves; the general choice
            // (extension operands, next tile: some 60 scalar instructions in front of a matrix instruction) is left to
            // the last slices of a tile, behind a branch that is rarely taken
            const bool tail = kt + 2 >= nfull;
            if (__builtin_expect(tail, 0)) select_slice(kt + 2);
            else src_so = (kt + 2) * (BK * 2);
            // W of slice g + 2 goes into the stage that slice g - 1 left at the previous barrier, six blocks before its
            // first fragment is read (issued in the second block: the first still sees the X loads of the block before it)
            block(IC<0>{}, IC<0>{}, IC<0>{}, cur, wst, IC<0>{}, 0);
            block(IC<1>{}, IC<1>{}, IC<1>{}, cur, wst, IC<1>{}, wst2);
            block(IC<0>{}, IC<1>{}, IC<0>{}, cur, wst, IC<0>{}, 0);
            // vmcnt(8) lgkmcnt(0): all but the eight W loads of this slice have landed (loads return in the order
            // issued), which is the whole of the next slice
            __builtin_amdgcn_s_waitcnt(0x0078);
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            // every wave has read this slice's X: X of slice g + 2 goes into its stage, three blocks ahead
            block(IC<1>{}, IC<0>{}, IC<1>{}, cur ^ 1, wst1, IC<2>{}, cur);
            wst = wst1;
        }
        // the tile's last matrix instruction has issued; the stages of slice g hold the next tile's first slice, fragment
        // set 0 its sub-step 0, and its second slice is in flight; W stage wst - 1 is idle until the next W loads
        const bool more = it + 1 < n_tiles;
        if constexpr (OUT == 1) {
            // A lane holds 16 consecutive outputs of one token per group of four blocks, so stored from the registers every
            // store touches 16 rows.  Instead each wave passes its 128 x 128 block through LDS, 32 tokens at a time, in its
            // quarter of the W stage that is idle between two tiles: written as held (16-byte chunk c of row t at
            // c ^ (t mod 16): the lanes of one write spread over all banks), read back 16 lanes to a 256-byte row, and
            // stored four whole rows to an instruction.
            asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7");     // (the matrix instructions are written out: their results' wait states too)
            char* stg = smem + W_BASE + ((wst == 0) ? 2 : wst - 1) * TILE_BYTES + wave * 8192;
#pragma clang loop unroll(full)
            for (int r2 = 0; r2 < 4; ++r2) {
#pragma clang loop unroll(full)
                for (int jj = 0; jj < 2; ++jj) {
                    const int J = 2 * r2 + jj, trow = jj * 16 + lc;
#pragma clang loop unroll(full)
                    for (int i4 = 0; i4 < 2; ++i4) {
                        uint32_t w[8];
#pragma clang loop unroll(full)
                        for (int t = 0; t < 4; ++t) {
                            const floatx4 v = acc[i4 * 4 + t][J];
                            w[2 * t] = pack_bf16x2(v[0], v[1]);
                            w[2 * t + 1] = pack_bf16x2(v[2], v[3]);
                        }
                        const int c0 = i4 * 8 + lg * 2;
                        *reinterpret_cast<uint4*>(stg + trow * 256 + ((c0 ^ (trow & 15)) << 4)) = make_uint4(w[0], w[1], w[2], w[3]);
                        *reinterpret_cast<uint4*>(stg + trow * 256 + (((c0 + 1) ^ (trow & 15)) << 4)) = make_uint4(w[4], w[5], w[6], w[7]);
                    }
                }
                const int cc = lane & 15;
#pragma clang loop unroll(full)
                for (int n = 0; n < 8; ++n) {
                    const int t = 4 * n + (lane >> 4);
                    const uint4 v = *reinterpret_cast<const uint4*>(stg + t * 256 + ((cc ^ (t & 15)) << 4));
                    *reinterpret_cast<uint4*>(reinterpret_cast<bf16_t*>(p.Y) + (m0 + wb * 128 + r2 * 32 + t) * p.ldy + n0 + wa * 128 + cc * 8) = v;
                }
            }
            __syncthreads();                                 // the next W loads go into that stage
            if (!more) break;
        } else if constexpr (OUT == 2) {
            // a lane holds 32 of the 128 logits of the wave's columns for each of eight tokens; the lanes lane ^ 16, ^ 32, ^ 48
            // hold the others.  Online softmax over the wave's 128 columns, per token
            asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7");
#pragma clang loop unroll(full)
            for (int J = 0; J < 8; ++J) {
                const int64_t row = m0 + wb * 128 + J * 16 + lc;
                const int tgt = p.ce_target[row];
                float mx = -INFINITY, tl = 0.f;
                bool has_tl = false;
#pragma clang loop unroll(full)
                for (int i4 = 0; i4 < 2; ++i4) {
                    const int trel = (tgt >= 0) ? (int)((int64_t)tgt - (n0 + wa * 128 + i4 * 64 + lg * 16)) : -1;
#pragma clang loop unroll(full)
                    for (int t = 0; t < 4; ++t)
#pragma clang loop unroll(full)
                        for (int e = 0; e < 4; ++e) {
                            const float y = acc[i4 * 4 + t][J][e];
                            mx = fmaxf(mx, y);
                            if (4 * t + e == trel) { tl = y; has_tl = true; }
                        }
                }
                mx = fmaxf(mx, __shfl_xor(mx, 16));
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                // exp(y - mx) as 2^((y - mx) log2 e) on the hardware exponential: the difference is exact enough in fp32
                // (one rounding), the terms that matter have small exponents, and the far tail underflows to 0
                float sm = 0.f;
#pragma clang loop unroll(full)
                for (int I = 0; I < 8; ++I)
#pragma clang loop unroll(full)
                    for (int e = 0; e < 4; ++e) sm += __builtin_amdgcn_exp2f((acc[I][J][e] - mx) * 1.44269504088896341f);
                sm += __shfl_xor(sm, 16);
                sm += __shfl_xor(sm, 32);
                const int64_t chunk = tn * 2 + wa;           // of tiles_n x 2 chunks per token
                if (lg == 0) p.ce_ms[chunk * p.M + row] = make_float2(mx, sm);
                if (has_tl) p.ce_tl[row] = tl;
            }
            if (!more) break;
        } else if constexpr (PHASES == 1) {
            const int64_t tm_done = tm, tn_done = tn;
            double part;
            if (more) {
                tile_at(it + 1, tm, tn);
                m0 = tm * BT; n0 = tn * BT;
                // The next tile's target is requested and the finished tile summed, in one order by two of the waves and in
                // the other by the other two: a request keeps its wave's issue port for as long as the address unit takes
                // over its 64 rows, and the address unit is the compute unit's one, so four waves requesting at once wait
                // for each other while nobody sums
                if (wave < 2) { request_target(); part = eval_sum(); }
                else { part = eval_sum(); request_target(); }
            } else {
                part = eval_sum();
            }
            eval_finish(part, 0, tm_done, tn_done, reinterpret_cast<double*>(smem + W_BASE + ((wst == 0) ? 2 : wst - 1) * TILE_BYTES));
            if (!more) break;
        } else {
            // shared forward: one tile per workgroup.  All LDS stages are free once the re-fetched slices have landed: the
            // first extension slice of each perturbed evaluation is requested before the evaluation that precedes it (X and
            // W stages 0 for +eps, 1 for -2 eps); further slices (r > 16) one at a time; the sums meet in W stage 2
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads();
            const __amdgpu_buffer_rsrc_t rx2 = rsrc(xb2), rw2 = rsrc(wb2), rw3 = rsrc(wb3);
            auto ext_dma = [&](const __amdgpu_buffer_rsrc_t& rws, int e, int buf) __attribute__((always_inline)) {
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const int t = q >> 1;
                    char* dst = smem + buf * TILE_BYTES + wave * 1024 + t * 4096 + ((q & 1) ? W_BASE : X_BASE);
                    if (q & 1) __builtin_amdgcn_raw_ptr_buffer_load_lds(rws, (lptr_t)dst, 16, vw2 + (t >> 1) * (2 * gs2) + (t & 1) * (gs2 >> 2), e * (BK * 2), 0, 0);
                    else __builtin_amdgcn_raw_ptr_buffer_load_lds(rx2, (lptr_t)dst, 16, vx2 + t * gs2, e * (BK * 2), 0, 0);
                }
            };
            if (next > 0) ext_dma(rw2, 0, 0);
            double* red = reinterpret_cast<double*>(smem + W_BASE + 2 * TILE_BYTES);
            evaluate(0, tm, tn, red);
            if (next > 0) {
                ext_dma(rw3, 0, 1);
                __builtin_amdgcn_s_waitcnt(0x0F70 | 16);     // the +eps slice has landed (the -2 eps one may be in flight)
                __syncthreads();
                multiply_slice(0, true);
                for (int e = 1; e < next; ++e) {
                    __syncthreads();
                    ext_dma(rw2, e, 0);
                    __builtin_amdgcn_s_waitcnt(0x0F70);
                    __syncthreads();
                    multiply_slice(0, true);
                }
            }
            evaluate(1, tm, tn, red);
            if (next > 0) {
                __builtin_amdgcn_s_waitcnt(0x0F70);
                __syncthreads();
                multiply_slice(1, true);
                for (int e = 1; e < next; ++e) {
                    __syncthreads();
                    ext_dma(rw3, e, 1);
                    __builtin_amdgcn_s_waitcnt(0x0F70);
                    __syncthreads();
                    multiply_slice(1, true);
                }
            }
            evaluate(2, tm, tn, red);
            break;
        }
        // ---- hand the accumulators to the next tile ----
        if constexpr (OUT != 0) {
            tile_at(it + 1, tm, tn);
            m0 = tm * BT; n0 = tn * BT;
        }
        tile_sources();
        next_sources(it + 2);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                      // the slices fetched past the end of the list
    if (p.clk && blockIdx.x == 0 && tid == 0) { p.clk[2] = __builtin_readcyclecounter(); p.clk[3] = wall_clock64(); }
}

template <int OUT, bool T_F32, int PHASES>
static hipError_t launch_aligned_variant(const GemmParams& p, hipStream_t st) {
    static bool attr_set = false;
    const int smem = 5 * TILE_BYTES;           // three W stages and two X stages: all 160 KiB of a compute unit's LDS
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_bf16_aligned_kernel<OUT, T_F32, PHASES>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    // one workgroup per compute unit, each with a list of tiles (a multiple of 8 workgroups: one share per XCD); the
    // shared-forward schedule needs both LDS stages between its evaluations and takes one tile per workgroup
    int64_t G = (int64_t)p.tiles_m * p.tiles_n;
    if (PHASES == 1) {
        int dev = 0, cus = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return e;
        if (cus < 1) return hipErrorInvalidDevice;
        if (G > cus) G = cus;
        if (G >= 8) G -= G % 8;
    }
    dim3 grid((unsigned)G);
    hipLaunchKernelGGL((gemm_bf16_aligned_kernel<OUT, T_F32, PHASES>), grid, dim3(256), smem, st, p);
    return hipGetLastError();
}

hipError_t launch_gemm_bf16_aligned(const GemmParams& p, hipStream_t st) {
    const bool shape_ok = p.vec_ok && p.M % BT == 0 && p.N % BT == 0 && p.K % BK == 0 && p.K >= 2 * BK &&
                          (p.P == nullptr || p.Xext != nullptr);
    if (!shape_ok) return hipErrorInvalidValue;
    if (p.Y != nullptr) {       // stored output, no loss
        if (p.loss_kind != AGZO_LOSS_NONE || p.y_dtype != AGZO_BF16 || p.shared) return hipErrorInvalidValue;
        return launch_aligned_variant<1, false, 1>(p, st);
    }
    if (p.loss_kind == AGZO_LOSS_CE) {
        if (p.shared || !p.ce_target || !p.ce_ms || !p.ce_tl) return hipErrorInvalidValue;
        return launch_aligned_variant<2, false, 1>(p, st);
    }
    if (p.loss_kind != AGZO_LOSS_MSE || (p.shared && p.Wext2 == nullptr)) return hipErrorInvalidValue;
    const bool f32 = p.target_dtype != AGZO_BF16;
    if (p.shared) return f32 ? launch_aligned_variant<0, true, 3>(p, st) : launch_aligned_variant<0, false, 3>(p, st);
    return f32 ? launch_aligned_variant<0, true, 1>(p, st) : launch_aligned_variant<0, false, 1>(p, st);
}

}  // namespace agzo
