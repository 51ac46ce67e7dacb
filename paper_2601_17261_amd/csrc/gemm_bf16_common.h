// Shared between the two tilings of the bf16 forward GEMM (gemm_bf16.hip: 256 x 256 tiles for shapes that fill the
// chip with them; gemm_bf16_small.hip: 128 x 128 tiles for the others): launch parameters and the LDS tile layout.
#pragma once
#include "agzo_internal.h"

namespace agzo {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
template <int V> struct IC { static constexpr int value = V; };

constexpr int BT = 256;                        // tile edge (tokens and outputs)
constexpr int BK = 64;
constexpr int CHUNKS = BK / 8;                 // 16-byte chunks per tile row
constexpr int TILE_BYTES = BT * BK * 2;        // one operand tile: 32 KiB

// byte offset of 16-byte chunk `c` of row `row` inside a [256][64] bf16 tile; the XOR spreads the
// 16 rows touched by one pass of a ds_read_b128 over all LDS banks.
__device__ __forceinline__ int lds_off(int row, int c) { return row * (BK * 2) + ((c ^ ((row >> 1) & 7)) << 4); }

// LDS row m' of a 32-row block holds W row perm(m'): MFMA output register e of lane half h is
// row 8*(e/4) + 4*h + e%4 of the block, which this makes output column 16*h + e.
__device__ __forceinline__ int w_perm(int m) { return ((m >> 2) & 1) * 16 + ((m >> 3) & 3) * 4 + (m & 3); }

struct GemmParams {
    const bf16_t* X; int64_t ldx;
    const bf16_t* W; int64_t ldw;
    int64_t M, N, K;            // tokens, outputs, d_in
    void* Y; int y_dtype; int64_t ldy;
    const float* P; int r; int rp;
    // rank-r extension operands prepared ahead of the launch (NULL: the workgroups build them per tile):
    // Xext [M][ext_ld] = [Ph | Ph | Pl | 0], Wext [N][ext_ld] = [Gh | Gl | Gh | 0] with the signed eps folded into G
    // Wext2: the W side once more with -2 eps folded in (second pass of the shared-forward squared-error kernel)
    const bf16_t* Xext; const bf16_t* Wext; const bf16_t* Wext2; int ext_ld;
    float eps_signed; uint32_t s_lo, s_hi;
    int loss_kind; int target_dtype; const void* target; int64_t ldt; double* partials;
    int tiles_m, tiles_n;
    int group_m;                // token tiles walked per output tile inside an XCD's run
    int vec_ok;                 // 16-byte epilogue accesses are legal
    int shared;                 // one pass evaluates f0, f+ and f- (three loss partials per tile)
    // cross-entropy: per (128-column chunk, token) running max and sum of exponentials, and the target's logit
    const int32_t* ce_target; float2* ce_ms; float* ce_tl;
    // fused range sketch (128 x 128 tiling only; NULL: none): Omega^T planes [3][16][sk_mpad] (sk_mpad a multiple of
    // 128 that covers every token tile, zero past the last token) and the per-token-tile partial sums [tiles_m][K][16]
    const bf16_t* sk_T; int64_t sk_mpad; float* sk_partial;
    // optional telemetry: workgroup 0 leaves {shader clock, constant-rate clock} at entry and at exit
    unsigned long long* clk;
};


// small-tile variant (gemm_bf16_small.hip): plain or perturbed forward with optional Y store and squared-error loss;
// partials [tiles128_m * tiles128_n]
constexpr int BT_SMALL = 128;
hipError_t launch_gemm_bf16_small(const GemmParams& p, hipStream_t st);

// kernel for tile-aligned layers (gemm_bf16_aligned.hip): M, N multiples of 256, d_in a multiple of 64 and >= 128,
// 16-byte target / output accesses, the rank-r term as prepared operands; either the squared-error loss without a
// stored Y (p.shared: f0, f+, f- in one pass, needs Wext2, partials [3][tiles]) or a bf16 Y without a loss
hipError_t launch_gemm_bf16_aligned(const GemmParams& p, hipStream_t st);

}  // namespace agzo
