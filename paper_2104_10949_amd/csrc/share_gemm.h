// Internal interface between the C-ABI entry points and the fused share-product kernel.
#ifndef CG_SHARE_GEMM_H
#define CG_SHARE_GEMM_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cg {

// Division of a 32-bit unsigned n < 2^31 by a run-time constant as multiply-high,
// add, shift (round-up method of Granlund and Montgomery).
struct FastDiv {
    uint32_t mul, shift;
};

inline FastDiv make_fast_div(uint32_t d) {
    FastDiv f;
    uint32_t s = 0;
    while ((1ull << s) < d) ++s;
    f.shift = s;
    f.mul = (uint32_t)((((1ull << s) - d) << 32) / d + 1);
    return f;
}

// The 32-channel patch gathers keep one bit per filter tap (inside the image or not) in a 32-bit register.
constexpr int MAX_MASK_TAPS = 32;

// How the left operand's words are addressed.
enum AMode {
    A_LINEAR_VEC = 0,     // row-major [M, lda], 16-byte loads (lda even, 16-byte aligned base)
    A_LINEAR_SCALAR = 1,  // row-major [M, lda], 8-byte loads
    A_CONV_C32 = 2,       // NHWC patch gather, Cin % 32 == 0, at most MAX_MASK_TAPS taps, 16-byte loads
    A_CONV_GEN = 3,       // NHWC patch gather, any Cin, 8-byte loads
    A_TRANS = 4,          // stored transposed, [K, M] with M contiguous, 8-byte loads
    A_CONV_DIL = 5,       // NHWC patch gather from an image whose pixels sit dil_h, dil_w apart
                          // with zeros between them (input gradient of a strided convolution)
    A_PLANES = 6,         // row-major [M, K] kept as digit planes (xp_a, xp_b; see to_planes_kernel)
    A_PLANES_CONV = 7,    // NHWC patch gather, Cin % 32 == 0, from the digit planes of the [pixels, Cin] matrix
    // Weight gradient with the operands exchanged: the left operand is the layer input, A[(r, s, c), pixel] =
    // patch entry (B_PATCH_T's generator), the right one the transposed gradient (B_TRANS), and z is written
    // transposed, z[col * M + row]: few output channels then fill the 64-column side of the tile.
    A_PATCH_T = 8,
    A_LINEAR_WIDE = 9     // row-major [M, lda] with rows too long for 32-bit offsets (256 rows of more than 2^31
                          // bytes): 64-bit addresses, 8-byte loads, explicit bounds
};

// How the right operand's words are addressed.
enum BMode {
    B_VEC = 0,     // row-major [N, K], 16-byte loads
    B_SCALAR = 1,  // row-major [N, K], 8-byte loads
    B_TRANS = 2,   // stored transposed, [K, N] with N contiguous, 8-byte loads
    // Input gradient of a convolution: the right operand is the filter [Cout, kh, kw, N] read as
    // B[n, (r', s', co)] = W[co, kh-1-r', kw-1-s', n].
    B_FLIP_C32 = 3,  // ... Cout % 32 == 0: a slice of K has one tap, rebased per slice; the window may
                     // cover a regular sub-grid of the filter's taps and the output rows a regular
                     // sub-grid of the pixels (see flt_* and out_* below)
    B_FLIP_GEN = 4,  // ... any Cout: every word finds its own tap
    // Weight gradient: the right operand is the layer input, B[(r, s, c), pixel] = patch entry
    B_PATCH_T = 5,
    B_PLANES = 6,    // row-major [N, K] kept as digit planes (wp_sum, wp_a)
    B_WIDE = 7       // row-major [N, K] with rows too long for 32-bit offsets (see A_LINEAR_WIDE)
};

struct GemmParams {
    const uint64_t *x_a, *x_b;  // left operand shares  s_i, s_{i+1}
    const uint64_t *w_a, *w_b;  // right operand shares s_i, s_{i+1}, [N, K] row-major
    uint64_t* z;                // [M, N] row-major
    int M, N, K;                // matrix-product view
    int lda;                    // leading dimension of the left operand (linear modes)
    uint64_t x_elems;           // words in one left-operand share tensor
    uint64_t w_elems;           // words in one right-operand share tensor
    uint64_t img_elems;         // H*W*Cin (patch modes)
    int H, W, Cin, Ho, Wo, kh, kw, sh, sw, ph, pw;
    FastDiv div_cin, div_kw;
    int dil_h, dil_w;           // A_CONV_DIL: spacing of the stored pixels inside the gathered image
    FastDiv div_dil_h, div_dil_w;
    FastDiv div_howo, div_wo;   // B_PATCH_T, B_FLIP_C32: decomposition of a pixel index into (b, ho, wo)
    // B_FLIP_C32: the filter's own tap grid is flt_kh x flt_kw; tap (r', s') of the gathered kh x kw window
    // reads filter tap (flt_r0 + flt_sh*(kh-1-r'), flt_s0 + flt_sw*(kw-1-s')).
    int flt_kh, flt_kw, flt_r0, flt_s0, flt_sh, flt_sw;
    // B_FLIP_C32: output row (b, i, j) of the [B, Ho, Wo] grid is pixel (out_h0 + out_sh*i, out_w0 + out_sw*j)
    // of the stored tensor z [B, out_H, out_W, N].
    int out_H, out_W, out_h0, out_w0, out_sh, out_sw;
    int z_prezeroed;            // the caller has cleared z: launches that add into z do not clear it again
    int z_add;                  // z holds a value on entry and the product is added to it
    // digit-plane route: planes of x_i, x_{i+1}, y_i + y_{i+1}, y_i (see to_planes_kernel)
    const char *xp_a, *xp_b, *wp_sum, *wp_a;
    uint64_t xp_bytes;          // bytes of one left-operand plane tensor
    uint64_t wp_bytes;          // bytes of one right-operand plane tensor
    int group_m;                // tile-rows per launch-order group (set by the launcher)
    int ksplit;                 // number of K ranges the grid is replicated over (set by the launcher)
    int64_t stream_per;         // > 0: (tile, slice) units per block of the streamed distribution (set by the launcher)
    // Divisors of the block's index arithmetic as multiply-shift pairs (set by the launcher from the tile shape
    // and the fields above): a block's first load waits for this arithmetic, and a division by a value known
    // only at run time is some thirty dependent instructions.
    FastDiv div_tiles;          // tiles of the launch (classic distribution: block -> (split, tile))
    int per_split;              // slices per K range of the classic distribution
    FastDiv div_per_group;      // group_m * tile columns
    FastDiv div_group, div_last_group;   // tile-rows of a full group / of the last, shorter one (or of a full one)
    FastDiv div_taps, div_tap_kw;        // kh * kw and kw, for the tap cursor
    FastDiv div_row_howo, div_row_wo;    // Ho * Wo and Wo, for the pixel of an output row
    uint32_t tap_rows;          // bit r*kw for every row r of the kh x kw tap grid (tap masks of the patch gathers)
};

// Largest block-tile height any instantiation uses; the host checks 32-bit
// offset ranges against it.
static const int MAX_TILE_ROWS = 256;

hipError_t launch_share_gemm(const GemmParams& p, int amode, int bmode, hipStream_t stream);

// Products with few rows on the left (share_gemm_small.hip): row-major operands that A_LINEAR_VEC / B_VEC
// address (K even, 16-byte aligned bases, lda == K).  `applies` says whether the launcher takes p.
bool share_gemm_small_applies(const GemmParams& p);
hipError_t launch_share_gemm_small(const GemmParams& p, hipStream_t stream);

// The same product of row-major x [M, K] and w [N, K] on the float64 matrix instruction with
// four 16-bit blocks per word (share_gemm_f64.hip); K below 2^31 / 8 words per row is the
// caller's business, the kernel indexes with 64-bit offsets.
hipError_t launch_share_gemm_f64limb(const uint64_t* x_a, const uint64_t* x_b, const uint64_t* w_a,
                                     const uint64_t* w_b, uint64_t* z, int M, int N, int K, hipStream_t stream);

// z[0..n) = 0 with a fill kernel (capturable).
hipError_t launch_zero_words(uint64_t* z, size_t n, hipStream_t stream);

// Digit-plane route.  launch_to_planes converts, in one launch, the four operands of p into the
// plane tensors p.xp_a, p.xp_b (left operand shares, seen as a row-major [x_rows, x_k] matrix),
// p.wp_sum (w_a + w_b) and p.wp_a (right operand, [N, K]); rows of K even, 16-byte aligned.  A
// row-major [R, K] operand takes planes_bytes(R, K) bytes.  launch_share_gemm with the modes
// A_PLANES / A_PLANES_CONV and B_PLANES then contracts the four plane tensors.
hipError_t launch_to_planes(const GemmParams& p, int64_t x_rows, int64_t x_k, hipStream_t stream);
inline uint64_t planes_bytes(int64_t R, int64_t K) {
    return (uint64_t)((R + 15) / 16 * 16) * (uint64_t)((K + 31) / 32) * 256u;
}

}  // namespace cg
#endif
