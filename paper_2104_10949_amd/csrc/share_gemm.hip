// One party's local product on replicated shares over Z_{2^64}, as one fused
// int8-MFMA kernel for gfx950 (CryptGPU Sec. III-B, "Multiplication" and
// "Convolutions and matrix multiplication").
//
// What is computed.  The party holds (x_a, x_b) = (x_i, x_{i+1}) and
// (w_a, w_b) = (y_i, y_{i+1}) and needs
//     z = x_a*w_a + x_b*w_a + x_a*w_b                    (mod 2^64).
// By distributivity this is x_a*(w_a + w_b) + x_b*w_a: two ring products, i.e.
// one matrix product over the doubled contraction length
//     [x_a | x_b] * [w_a + w_b | w_a]^T.
// A matrix instruction contracts 64 bytes; here these are one digit of a 32-word
// slice of K for BOTH terms at once: [x_a | x_b] against [w_a + w_b | w_a].
//
// How a ring product runs on the matrix cores.  A 64-bit word a is rewritten
// as eight SIGNED byte digits d_0..d_7 in [-128,127] with
// a = sum_l d_l 2^(8l) (mod 2^64); the closed form is
// t = (a + 0x8080808080808080) ^ 0x8080808080808080, d_l = (int8) byte l of t.
// (Sec. II-B uses the same idea with four unsigned 16-bit blocks fed to float64
// kernels; bytes are what the int8 MFMA of CDNA4 consumes.)  Then
//     a*b = sum_{l+m<=7} d_l(a) d_m(b) 2^(8(l+m))        (mod 2^64),
// 36 digit pairs; pairs with l+m >= 8 vanish mod 2^64 (Sec. II-B: only block
// products with w(i+j-2) < 64 are needed).  All pairs with the same s = l+m
// share one i32 accumulator P_s, so a 32x32 output tile keeps eight of them.
// |d d'| <= 2^14, and P_s receives (s+1)*64 products per slice, so P_0..P_3
// stay exact in i32 for 511 slices; P_4..P_7 only matter mod 2^(64-8s) <=
// 2^32, where i32 wraparound (verified on hardware) is harmless.  After at most
// SEG_KSTEPS slices of K the accumulators are folded into the 64-bit result
// z += sum_s sext(P_s) << 8s and cleared.
//
// Data movement.  Each share tile is read from HBM once per block as raw
// uint64 (coalesced 16-byte buffer loads, out-of-range lanes return 0, which
// is exact padding in the ring), split into digit planes in registers
// (4 integer ops + 4 byte permutes per word), written to LDS as
// [digit][k-group][row][16 bytes] so that every MFMA operand is one conflict-free
// ds_read_b128, and consumed by v_mfma_i32_16x16x64_i8.  Convolution and the
// backward products of both layer kinds (Sec. III-C) use the same kernel: only the
// address generators of the operands differ (patch gather from NHWC with zero
// fill, operands stored transposed, the filter read with its taps reversed, patch
// entries gathered as the right operand).  Nothing but z is written to HBM.
//
// build.py compiles the file three times, with -DCG_INST_GROUP=0, 1, 2: every group instantiates the kernel for a
// third of the address-generator pairs (see launch_share_gemm at the end), so that the three compile side by side;
// group 0 also holds the conversion and clearing kernels and the entry point itself.  Without the macro the file
// compiles to one object with everything.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "share_digits.h"
#include "share_gemm.h"

#ifdef CG_INST_GROUP
#define CG_G0 (CG_INST_GROUP == 0)
#define CG_G1 (CG_INST_GROUP == 1)
#define CG_G2 (CG_INST_GROUP == 2)
#else   // compiled on its own: everything in one object
#define CG_G0 1
#define CG_G1 1
#define CG_G2 1
#endif

namespace cg {

// Slices of K (32 words of each share) between two folds of the i32 accumulators: a slice adds
// (s + 1) * 64 digit products of at most 2^14 to P_s, so P_0..P_3 stay exact for 511 slices.
static constexpr int SEG_KSTEPS = 511;

// Block tile of the fused kernel: WM x WN waves, each computing a 32 x 32 sub-tile as 2 x 2 blocks of
// v_mfma_i32_16x16x64_i8.  One step covers a 32-word slice of K for BOTH shares of each operand:
// the 64 contraction bytes of an instruction are [x_a | x_b] against [w_a + w_b | w_a], 16 bytes per
// "k-group" (two halves of the slice times two shares).  LDS holds digit planes
//     [digit][k-group 4][row][16 bytes]
// for the left operand in two parts, digits 0-3 (two buffers) and digits 4-7 (one buffer), and for
// the right operand in two buffers of all eight digits: 3*A_HALF + 2*B_ALL bytes (160 KB at 128 x 64).
template <int WM_, int WN_>
struct StepTile {
    static constexpr int WM = WM_, WN = WN_;
    static constexpr int BM = WM * 32, BN = WN * 32;
    static constexpr int NT = WM * WN * 64;
    // A "unit" is 4 words of one row of one share: two 16-byte loads, eight 4-byte LDS writes.
    static constexpr int A_UNITS = BM * 8 / NT, B_UNITS = BN * 8 / NT;
    static constexpr int A_RS = BM * 16, B_RS = BN * 16;      // one [digit][k-group] slab
    static constexpr int A_DIG = 4 * A_RS, B_DIG = 4 * B_RS;  // one digit
    static constexpr int A_HALF = 4 * A_DIG, B_ALL = 8 * B_DIG;
    static constexpr int OFF_AHI = 2 * A_HALF, OFF_B = 3 * A_HALF;
    static constexpr int LDS_BYTES = 3 * A_HALF + 2 * B_ALL;
    static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile does not divide over the threads");
    static_assert(LDS_BYTES <= 160 * 1024, "tile does not fit the LDS of a compute unit");
    static_assert(3 * A_DIG + 256 < 65536 && 7 * B_DIG + 256 < 65536, "fragment offsets must fit an LDS immediate");
};
typedef StepTile<4, 2> DefaultStepTile;

__device__ __forceinline__ u32 fast_div(u32 n, FastDiv d) {
    return ((u32)(((u64)n * d.mul) >> 32) + n) >> d.shift;
}

// Four words (two 16-byte registers) -> eight digit dwords, written to the slab
// set starting at `dst` (byte address of digit 0 for this unit's row/k slot).
template <int RS>
__device__ __forceinline__ void split_store(u4 v0, u4 v1, char* dst) {
    u32 lo[4] = {v0.x, v0.z, v1.x, v1.z}, hi[4] = {v0.y, v0.w, v1.y, v1.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) recode(lo[i], hi[i]);
    u32 d[8];
    transpose4(lo[0], lo[1], lo[2], lo[3], d);
    transpose4(hi[0], hi[1], hi[2], hi[3], d + 4);
#pragma unroll
    for (int l = 0; l < 8; ++l) *reinterpret_cast<u32*>(dst + l * 2 * RS) = d[l];
}

__device__ __forceinline__ u4 add64x2(u4 a, u4 b) {
    const u64 s0 = (((u64)a.y << 32) | a.x) + (((u64)b.y << 32) | b.x);
    const u64 s1 = (((u64)a.w << 32) | a.z) + (((u64)b.w << 32) | b.z);
    u4 r;
    r.x = (u32)s0; r.y = (u32)(s0 >> 32); r.z = (u32)s1; r.w = (u32)(s1 >> 32);
    return r;
}

// ---------------------------------------------------------------------------
// Address generators.  A unit is identified by (row, q, jh): row inside the
// block tile, q = which 16-byte quarter of a 64-byte group, jh = which half of
// the 32-word slice.  Its two loads jj = 0,1 fetch words
//     k = 32*ks + 16*jh + 8*jj + 2*q + {0,1}.
// The same (jh, q, jj) -> LDS byte slot map is used for both operands, which is
// all the contraction needs: digit bytes meet their partner, in any order.
// An offset of OOB or more is outside every view, so "OOB + something small"
// still reads zeros: invalid rows need no per-load select.
// ---------------------------------------------------------------------------

// Row-major [rows, ld] operand, 16-byte loads (ld even, base 16-byte aligned).
struct LinearVec {
    u32 off0;  // byte offset of word k = 16*jh + 2*q of the row inside the view, or OOB
    u32 kq;    // 16*jh + 2*q
    __device__ __forceinline__ void init(const GemmParams&, int, int row_local, int rows_left, u32 ld,
                                         int q, int jh) {
        kq = 16 * jh + 2 * q;
        off0 = row_local < rows_left ? (u32)row_local * ld * 8u + kq * 8u : OOB;
    }
    __device__ __forceinline__ void load(const GemmParams&, __amdgpu_buffer_rsrc_t r, int ks, u32 K,
                                         u4 out[2]) const {
        const u32 off = off0 + 256u * ks;
        const u32 k = 32u * ks + kq;
        out[0] = __builtin_amdgcn_raw_buffer_load_b128(r, k < K ? off : OOB, 0, 0);
        out[1] = __builtin_amdgcn_raw_buffer_load_b128(r, k + 8u < K ? off + 64u : OOB, 0, 0);
    }
};

// Row-major operand with 8-byte loads: any ld, any 8-byte-aligned base.
struct LinearScalar {
    u32 off0;
    u32 kq;
    __device__ __forceinline__ void init(const GemmParams&, int, int row_local, int rows_left, u32 ld,
                                         int q, int jh) {
        kq = 16 * jh + 2 * q;
        off0 = row_local < rows_left ? (u32)row_local * ld * 8u + kq * 8u : OOB;
    }
    __device__ __forceinline__ void load(const GemmParams&, __amdgpu_buffer_rsrc_t r, int ks, u32 K,
                                         u4 out[2]) const {
        const u32 off = off0 + 256u * ks;
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const u32 k = 32u * ks + kq + 8u * jj;
            const u2 e0 = __builtin_amdgcn_raw_buffer_load_b64(r, k < K ? off + 64u * jj : OOB, 0, 0);
            const u2 e1 = __builtin_amdgcn_raw_buffer_load_b64(r, k + 1 < K ? off + 64u * jj + 8u : OOB, 0, 0);
            out[jj].x = e0.x; out[jj].y = e0.y; out[jj].z = e1.x; out[jj].w = e1.y;
        }
    }
};

// Row-major operand whose rows are too long for the 32-bit offsets of a buffer view (a tile's 256 rows must
// stay below 2^31 bytes, i.e. ld <= 2^20 words): 64-bit addresses and 8-byte loads.  Nothing checks a range in
// hardware here, so a word outside the operand (rows past the end, the K tail, a loader past the block's range)
// is read from a word of zeros instead.
static __device__ u64 wide_zero_word[2];   // zero-initialised, never written (one copy per compiled group)

struct LinearWide {
    u64 row_w;  // word offset of word k = 16*jh + 2*q of the row, relative to the tile's first row
    u32 kq;
    bool ok;
    __device__ __forceinline__ void init(const GemmParams&, int, int row_local, int rows_left, u32 ld,
                                         int q, int jh) {
        kq = 16 * jh + 2 * q;
        ok = row_local < rows_left;
        row_w = (u64)row_local * (u64)ld + kq;
    }
    // `tile`: first word of the tile's first row in this share tensor; null for a loader past its range
    __device__ __forceinline__ void load_wide(const u64* tile, int ks, u32 K, u4 out[2]) const {
        const u64* src = tile + row_w + 32u * (u32)ks;
        const bool live = ok && tile != nullptr;
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const u32 k = 32u * ks + kq + 8u * jj;
            const u2 e0 = *reinterpret_cast<const u2*>(live && k < K ? src + 8 * jj : wide_zero_word);
            const u2 e1 = *reinterpret_cast<const u2*>(live && k + 1 < K ? src + 8 * jj + 1 : wide_zero_word);
            out[jj].x = e0.x; out[jj].y = e0.y; out[jj].z = e1.x; out[jj].w = e1.y;
        }
    }
};

// Transposed operand: memory holds [K, rows] with the rows contiguous (the operand of
// a backward-pass product).  Consecutive lanes take consecutive rows, so each of the
// unit's four 8-byte loads is one contiguous run per wave.  The view is rebased at
// every K slice (offsets inside a slice stay below 32 * pitch * 8 bytes).
struct TransScalar {
    u32 off0;  // (row + (16*jh + 2*q) * pitch) * 8, or OOB
    u32 kq, pitch8;
    __device__ __forceinline__ void init(const GemmParams&, int, int row_local, int rows_left, u32 pitch,
                                         int q, int jh) {
        kq = 16 * jh + 2 * q;
        pitch8 = pitch * 8u;
        off0 = row_local < rows_left ? ((u32)row_local + kq * pitch) * 8u : OOB;
    }
    __device__ __forceinline__ void load(const GemmParams&, __amdgpu_buffer_rsrc_t r, int ks, u32 K,
                                         u4 out[2]) const {
        // The four offsets are one add away from off0.  Hidden from the optimiser, the pitch keeps them from
        // being computed ahead of the loop and held in four registers per unit for its whole length.
        u32 p8 = pitch8;
        asm volatile("" : "+s"(p8));
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const u32 k = 32u * ks + kq + 8u * jj;
            const u32 o = off0 + 8u * jj * p8;
            const u2 e0 = __builtin_amdgcn_raw_buffer_load_b64(r, k < K ? o : OOB, 0, 0);
            const u2 e1 = __builtin_amdgcn_raw_buffer_load_b64(r, k + 1 < K ? o + p8 : OOB, 0, 0);
            out[jj].x = e0.x; out[jj].y = e0.y; out[jj].z = e1.x; out[jj].w = e1.y;
        }
    }
};

// Decomposition of an output-pixel row index shared by both patch gatherers.
// Offsets are 32-bit unsigned and may wrap for taps that fall outside the image;
// those are never used (the load is redirected to OOB).
struct PatchRow {
    u32 base;   // byte offset of pixel (hi0, wi0), channel 0, relative to the view (mod 2^32)
    int hi0, wi0;
    bool ok;
    __device__ __forceinline__ void init(const GemmParams& p, int m0, int row_local, int rows_left) {
        ok = row_local < rows_left;
        const u32 m = (u32)(m0 + (ok ? row_local : 0));
        const u32 HoWo = (u32)(p.Ho * p.Wo);
        const u32 b = fast_div(m, p.div_row_howo), b0 = fast_div((u32)m0, p.div_row_howo);
        const u32 rem = m - b * HoWo;
        const u32 ho = fast_div(rem, p.div_row_wo), wo = rem - ho * (u32)p.Wo;
        hi0 = (int)ho * p.sh - p.ph;
        wi0 = (int)wo * p.sw - p.pw;
        base = (b - b0) * (u32)p.H * (u32)p.W * (u32)p.Cin * 8u +
               ((u32)hi0 * (u32)p.W + (u32)wi0) * (u32)p.Cin * 8u;
    }
};

// Order of the contraction when Cin % 32 == 0.  A 32-word slice never straddles a
// filter tap, and the order of the slices is free as long as both operands follow it,
// so the slices are taken channel block by channel block, all taps of one block of 32
// channels before the next block.  The taps of one channel block read overlapping
// pixels, so a tile's working set between two uses of the same input word is one
// 32-channel block of its input rows instead of the whole rows: it stays in the L2
// cache of the tile's XCD, and every input word is fetched from memory about once
// instead of once per tap.  Slice ks of the loop is slice `pks` of the filter's own
// (tap, channel) order.  (r, s), c0 are uniform over the block and advance by scalar
// increments.
struct TapCursor {
    int ks, r, s, c0;   // the cursor proper; everything else is derived on use, to keep few values alive
    // put the cursor on slice `at` (once per tile)
    __device__ __forceinline__ void set(const GemmParams& p, int at) {
        const int taps = p.kh * p.kw;
        const int cb = (int)fast_div((u32)at, p.div_taps), t = at - cb * taps;
        ks = at; c0 = 32 * cb; r = (int)fast_div((u32)t, p.div_tap_kw); s = t - r * p.kw;
    }
    // `want` is the cursor's slice or the next one (the loaders move one slice at a time).  Written as selects:
    // branches here end up inside the K loop, where each costs the wave an instruction-fetch bubble and the
    // compiler a conservative wait at the join.
    __device__ __forceinline__ void advance_to(const GemmParams& p, int want) {
        const int d = want - ks;   // 0 or 1
        ks = want;
        s += d;
        const bool row_done = s == p.kw;
        s = row_done ? 0 : s;
        r += row_done ? 1 : 0;
        const bool block_done = r == p.kh;
        r = block_done ? 0 : r;
        c0 += block_done ? 32 : 0;   // past the end of K: c0 >= Cin
    }
    __device__ __forceinline__ int tap(const GemmParams& p) const { return r * p.kw + s; }
    // slice index in the filter's own (tap, channel) order
    __device__ __forceinline__ int pks(const GemmParams& p) const { return (tap(p) * p.Cin + c0) >> 5; }
    // ((r*W + s)*Cin + c0) * 8: byte offset of the slice relative to the row's pixel (hi0, wi0)
    __device__ __forceinline__ u32 off(const GemmParams& p) const {
        return (((u32)r * (u32)p.W + (u32)s) * (u32)p.Cin + (u32)c0) * 8u;
    }
};

// Bits [lo, hi) of a 32-bit word, 0 <= lo, hi <= 32 (empty when hi <= lo).
__device__ __forceinline__ u32 bit_range(int lo, int hi) {
    const u32 below_hi = hi >= 32 ? 0xFFFFFFFFu : (1u << hi) - 1u;
    const u32 below_lo = lo >= 32 ? 0xFFFFFFFFu : (1u << lo) - 1u;
    return hi > lo ? below_hi & ~below_lo : 0u;
}
// Which taps t = r*kw + s of a kh x kw window (at most 32 taps) whose corner sits on pixel (hi0, wi0) read a pixel
// inside the H x W image: rows r with 0 <= hi0 + r < H times columns s with 0 <= wi0 + s < W.  The valid columns
// are one run of bits, the valid rows select every kw-th bit of p.tap_rows: their product is the mask (the runs
// do not overlap), without a loop over the taps.
__device__ __forceinline__ u32 taps_inside(const GemmParams& p, int hi0, int wi0) {
    const int r_lo = hi0 < 0 ? -hi0 : 0, r_hi = p.H - hi0 < p.kh ? p.H - hi0 : p.kh;
    const int s_lo = wi0 < 0 ? -wi0 : 0, s_hi = p.W - wi0 < p.kw ? p.W - wi0 : p.kw;
    if (r_hi <= r_lo || s_hi <= s_lo) return 0u;   // (a select: both sides are a few instructions)
    const u32 rows = p.tap_rows & bit_range(r_lo * p.kw, r_hi * p.kw);
    return rows * bit_range(s_lo, s_hi);
}

// Patch gather with Cin % 32 == 0, 16-byte loads.  Which filter taps fall inside the image for this unit's
// output pixel is decided once, as a bit mask over the taps; the host sends windows of more than
// MAX_MASK_TAPS taps to the general gather.  Two registers per unit stay alive across the K loop.
struct ConvC32 {
    u32 base_kq;  // byte offset of word 16*jh + 2*q of pixel (hi0, wi0), relative to the view (mod 2^32)
    u32 inside;   // bit t: tap t = r*kw + s reads a pixel inside the image
    __device__ __forceinline__ void init(const GemmParams& p, int m0, int row_local, int rows_left, u32,
                                         int q, int jh) {
        PatchRow pr;
        pr.init(p, m0, row_local, rows_left);
        base_kq = pr.base + (u32)(16 * jh + 2 * q) * 8u;
        inside = pr.ok ? taps_inside(p, pr.hi0, pr.wi0) : 0u;
    }
    __device__ __forceinline__ void load(const GemmParams& p, __amdgpu_buffer_rsrc_t rs_, const TapCursor& t,
                                         u4 out[2]) const {
        const bool v = (t.c0 < p.Cin) & (((inside >> t.tap(p)) & 1) != 0);   // (no short circuit: no branch)
        u32 in_off = base_kq + t.off(p);
        asm volatile("" : "+v"(in_off));   // computed by every lane, then selected: no masked-off region in the K loop
        const u32 off = v ? in_off : OOB;
        out[0] = __builtin_amdgcn_raw_buffer_load_b128(rs_, off, 0, 0);
        out[1] = __builtin_amdgcn_raw_buffer_load_b128(rs_, off + 64u, 0, 0);
    }
};

// Patch gather, any Cin: every word finds its own tap; 8-byte loads.
struct ConvGen {
    PatchRow pr;
    u32 kq;
    __device__ __forceinline__ void init(const GemmParams& p, int m0, int row_local, int rows_left, u32,
                                         int q, int jh) {
        pr.init(p, m0, row_local, rows_left);
        kq = 16 * jh + 2 * q;
    }
    __device__ __forceinline__ u2 one(const GemmParams& p, __amdgpu_buffer_rsrc_t rs_, u32 k) const {
        const u32 rs = fast_div(k, p.div_cin);
        const u32 c = k - rs * (u32)p.Cin;
        const u32 r = fast_div(rs, p.div_kw);
        const u32 s = rs - r * (u32)p.kw;
        const bool v = pr.ok && k < (u32)p.K && (u32)(pr.hi0 + (int)r) < (u32)p.H &&
                       (u32)(pr.wi0 + (int)s) < (u32)p.W;
        const u32 off = pr.base + ((r * (u32)p.W + s) * (u32)p.Cin + c) * 8u;
        return __builtin_amdgcn_raw_buffer_load_b64(rs_, v ? off : OOB, 0, 0);
    }
    __device__ __forceinline__ void load(const GemmParams& p, __amdgpu_buffer_rsrc_t rs_, int ks, u32,
                                         u4 out[2]) const {
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const u32 k = 32u * ks + kq + 8u * jj;
            const u2 e0 = one(p, rs_, k), e1 = one(p, rs_, k + 1);
            out[jj].x = e0.x; out[jj].y = e0.y; out[jj].z = e1.x; out[jj].w = e1.y;
        }
    }
};

// Patch gather from a zero-interleaved image (any channel count, 8-byte loads).  The
// gathered image is the stored [H, W, Cin] tensor with dil_h - 1 rows and dil_w - 1
// columns of zeros between neighbouring pixels: position (hd, wd) holds stored pixel
// (hd / dil_h, wd / dil_w) when both divisions are exact and is zero otherwise.  This is
// what the input gradient of a strided convolution correlates the filter with.
struct ConvDil {
    u32 img_off;  // byte offset of this row's image relative to the view
    int hi0, wi0;
    bool ok;
    u32 kq;
    __device__ __forceinline__ void init(const GemmParams& p, int m0, int row_local, int rows_left, u32,
                                         int q, int jh) {
        ok = row_local < rows_left;
        const u32 m = (u32)(m0 + (ok ? row_local : 0));
        const u32 HoWo = (u32)(p.Ho * p.Wo);
        const u32 b = fast_div(m, p.div_row_howo), b0 = fast_div((u32)m0, p.div_row_howo);
        const u32 rem = m - b * HoWo;
        const u32 ho = fast_div(rem, p.div_row_wo), wo = rem - ho * (u32)p.Wo;
        hi0 = (int)ho * p.sh - p.ph;
        wi0 = (int)wo * p.sw - p.pw;
        img_off = (b - b0) * (u32)p.H * (u32)p.W * (u32)p.Cin * 8u;
        kq = 16 * jh + 2 * q;
    }
    __device__ __forceinline__ u2 one(const GemmParams& p, __amdgpu_buffer_rsrc_t rs_, u32 k) const {
        const u32 rs = fast_div(k, p.div_cin);
        const u32 c = k - rs * (u32)p.Cin;
        const u32 r = fast_div(rs, p.div_kw);
        const u32 s = rs - r * (u32)p.kw;
        const int hd = hi0 + (int)r, wd = wi0 + (int)s;
        // negative positions wrap to huge unsigned values and fail the range test below
        const u32 hq = fast_div((u32)hd & 0x7FFFFFFFu, p.div_dil_h), wq = fast_div((u32)wd & 0x7FFFFFFFu, p.div_dil_w);
        const bool v = ok && k < (u32)p.K && hd >= 0 && wd >= 0 && hq < (u32)p.H && wq < (u32)p.W &&
                       hq * (u32)p.dil_h == (u32)hd && wq * (u32)p.dil_w == (u32)wd;
        const u32 off = img_off + ((hq * (u32)p.W + wq) * (u32)p.Cin + c) * 8u;
        return __builtin_amdgcn_raw_buffer_load_b64(rs_, v ? off : OOB, 0, 0);
    }
    __device__ __forceinline__ void load(const GemmParams& p, __amdgpu_buffer_rsrc_t rs_, int ks, u32,
                                         u4 out[2]) const {
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const u32 k = 32u * ks + kq + 8u * jj;
            const u2 e0 = one(p, rs_, k), e1 = one(p, rs_, k + 1);
            out[jj].x = e0.x; out[jj].y = e0.y; out[jj].z = e1.x; out[jj].w = e1.y;
        }
    }
};

// Right operand of the input gradient, any Cout: word (n, k) with k = (r', s', co) is
// W[co, kh-1-r', kw-1-s', n] of the filter [Cout, kh, kw, N].  The view starts at column
// n0 of the filter and covers the rest of it (the host keeps a filter below 2^31 bytes).
struct FlipGen {
    u32 row8, kq;
    bool ok;
    __device__ __forceinline__ void init(const GemmParams&, int, int row_local, int rows_left, u32,
                                         int q, int jh) {
        kq = 16 * jh + 2 * q;
        ok = row_local < rows_left;
        row8 = (u32)row_local * 8u;
    }
    __device__ __forceinline__ u2 one(const GemmParams& p, __amdgpu_buffer_rsrc_t rs_, u32 k) const {
        const u32 taps = (u32)(p.kh * p.kw);
        const u32 tap = fast_div(k, p.div_cin);       // p.Cin is the gathered channel count = Cout
        const u32 co = k - tap * (u32)p.Cin;
        const bool v = ok && k < (u32)p.K;
        const u32 off = (co * taps + (taps - 1u - tap)) * (u32)p.N * 8u + row8;
        return __builtin_amdgcn_raw_buffer_load_b64(rs_, v ? off : OOB, 0, 0);
    }
    __device__ __forceinline__ void load(const GemmParams& p, __amdgpu_buffer_rsrc_t rs_, int ks, u32,
                                         u4 out[2]) const {
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const u32 k = 32u * ks + kq + 8u * jj;
            const u2 e0 = one(p, rs_, k), e1 = one(p, rs_, k + 1);
            out[jj].x = e0.x; out[jj].y = e0.y; out[jj].z = e1.x; out[jj].w = e1.y;
        }
    }
};

// Right operand of the weight gradient: row n = (r, s, c) of the filter layout, column
// k = output pixel (b, ho, wo); the word is X[b, ho*sh - ph + r, wo*sw - pw + s, c] or zero
// outside the image.  Consecutive lanes take consecutive n, i.e. consecutive channels of
// one pixel.  The view is rebased at every K slice to the image of the slice's first pixel.
struct PatchTrans {
    int r, s;
    u32 c8, kq;
    bool ok;
    __device__ __forceinline__ void init(const GemmParams& p, int n0, int row_local, int rows_left, u32,
                                         int q, int jh) {
        kq = 16 * jh + 2 * q;
        ok = row_local < rows_left;
        const u32 n = (u32)(n0 + (ok ? row_local : 0));
        const u32 tap = fast_div(n, p.div_cin);
        c8 = (n - tap * (u32)p.Cin) * 8u;
        r = (int)fast_div(tap, p.div_kw);
        s = (int)tap - r * p.kw;
    }
    __device__ __forceinline__ u2 one(const GemmParams& p, __amdgpu_buffer_rsrc_t rs_, u32 k, u32 b0) const {
        const u32 b = fast_div(k, p.div_howo);
        const u32 rem = k - b * (u32)(p.Ho * p.Wo);
        const u32 ho = fast_div(rem, p.div_wo), wo = rem - ho * (u32)p.Wo;
        const int hi = (int)ho * p.sh - p.ph + r, wi = (int)wo * p.sw - p.pw + s;
        const bool v = ok && k < (u32)p.K && (u32)hi < (u32)p.H && (u32)wi < (u32)p.W;
        const u32 off = ((((b - b0) * (u32)p.H + (u32)hi) * (u32)p.W + (u32)wi) * (u32)p.Cin) * 8u + c8;
        return __builtin_amdgcn_raw_buffer_load_b64(rs_, v ? off : OOB, 0, 0);
    }
    __device__ __forceinline__ void load(const GemmParams& p, __amdgpu_buffer_rsrc_t rs_, int ks, u32,
                                         u4 out[2]) const {
        const u32 b0 = fast_div(32u * (u32)ks, p.div_howo);  // the image the slice's view starts at
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const u32 k = 32u * ks + kq + 8u * jj;
            const u2 e0 = one(p, rs_, k, b0), e1 = one(p, rs_, k + 1, b0);
            out[jj].x = e0.x; out[jj].y = e0.y; out[jj].z = e1.x; out[jj].w = e1.y;
        }
    }
};

// Digit planes (see to_planes_kernel): this thread's row of a tile and its first piece.  The thread moves the
// pieces of ONE row: for the left operand those of digits cq and cq + 4 in both k-halves, for the right operand
// those of digit cq in both k-halves.
struct PlanesRow {
    u32 off0;  // byte offset, relative to the view, of piece cq of slice 0 of the row's 16-row block; or OOB
    __device__ __forceinline__ void init(int row_local, int rows_left, u32 KS, int cq) {
        off0 = row_local < rows_left
                   ? ((u32)(row_local >> 4) * KS * 16u + (u32)cq) * 256u + (u32)(row_local & 15) * 16u
                   : OOB;
    }
};

// Patch gather from the digit planes of the activations seen as a [pixels, Cin] matrix, Cin % 32 == 0, at most
// MAX_MASK_TAPS taps.
struct PlanesPatch {
    u32 pix0;     // pixel index of (hi0, wi0) relative to the view's first 16-pixel block (mod 2^32)
    u32 inside;   // bit t: tap t = r*kw + s reads a pixel inside the image
    u32 cq256;
    __device__ __forceinline__ void init(const GemmParams& p, int m0, int row_local, int rows_left, int cq) {
        const bool ok = row_local < rows_left;
        const u32 m = (u32)(m0 + (ok ? row_local : 0));
        const u32 HoWo = (u32)(p.Ho * p.Wo), HW = (u32)(p.H * p.W);
        const u32 b = fast_div(m, p.div_row_howo), b0 = fast_div((u32)m0, p.div_row_howo);
        const u32 rem = m - b * HoWo;
        const u32 ho = fast_div(rem, p.div_row_wo), wo = rem - ho * (u32)p.Wo;
        const int hi0 = (int)ho * p.sh - p.ph, wi0 = (int)wo * p.sw - p.pw;
        // the view starts at the 16-pixel block that holds the first pixel of image b0
        pix0 = ((b0 * HW) & 15u) + (b - b0) * HW + (u32)hi0 * (u32)p.W + (u32)wi0;
        cq256 = (u32)cq * 256u;
        inside = ok ? taps_inside(p, hi0, wi0) : 0u;
    }
    // byte offset of piece cq of the slice the cursor points at, or OOB
    __device__ __forceinline__ u32 offset(const GemmParams& p, const TapCursor& t) const {
        const bool v = (t.c0 < p.Cin) & (((inside >> t.tap(p)) & 1) != 0);   // (no short circuit: no branch)
        const u32 pix = pix0 + (u32)t.r * (u32)p.W + (u32)t.s;
        const u32 KS = (u32)p.Cin >> 5;
        u32 in_off = ((pix >> 4) * KS + ((u32)t.c0 >> 5)) * 4096u + cq256 + (pix & 15u) * 16u;
        asm volatile("" : "+v"(in_off));   // computed by every lane, then selected: no masked-off region in the K loop
        return v ? in_off : OOB;
    }
};

// compile-time loop: f(integral_constant<int, I>) for I in [I0, N)
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

__device__ __forceinline__ void recode2(u4& v) {
    u32 a = v.x, b = v.y, c = v.z, d = v.w;
    recode(a, b);
    recode(c, d);
    v.x = a; v.y = b; v.z = c; v.w = d;
}

// Work distribution.  The work of a launch is the list of (output tile, K slice) units in the
// launch order (group of group_m tile-rows, tile column, tile-row inside the group, slice), and
// every block takes one contiguous range of it:
//  * classic: the grid holds ksplit blocks per tile, block (split, tile) takes that tile's
//    split-th range of slices;
//  * streamed (p.stream_per > 0): one block per compute unit takes stream_per consecutive units,
//    whatever tiles they belong to, so the units are spread evenly even when the tile count is
//    just above a multiple of the number of compute units.  Partial tiles add into a cleared
//    output (ksplit > 1); when stream_per is a multiple of the slices of a tile every block
//    holds whole tiles and stores them plainly (ksplit == 1).  Either way the LDS pipeline of
//    a block runs on from one tile of its range into the next.
// The hardware deals consecutive block ids to the 8 XCDs in turn, and each XCD has an L2 cache of
// its own, so block ids are mapped such that every XCD works through one contiguous run of the
// order above (K splits slowest in the classic scheme).  With 8 or more splits an XCD therefore
// sees only its own ranges of K and reads its share of both operands once; with fewer, its run is
// a box of tile-rows times tile columns whose shape the host picks through group_m.
__device__ __forceinline__ int run_index(int total) {
    const int bid = blockIdx.x, xcd = bid & 7, idx = bid >> 3;
    const int per = total >> 3, rem = total & 7;
    return xcd * per + (xcd < rem ? xcd : rem) + idx;
}

__device__ __forceinline__ void logical_to_tile(const GemmParams& p, int tiles_m, int tiles_n, int logical, int& tm,
                                                int& tn) {
    const int GM = p.group_m;
    const int per_group = GM * tiles_n;
    const int g = (int)fast_div((u32)logical, p.div_per_group), in_g = logical - g * per_group;
    const int first = g * GM;
    const bool last = tiles_m - first < GM;   // the last group may hold fewer tile-rows
    const int gsz = last ? tiles_m - first : GM;
    FastDiv d;
    d.mul = last ? p.div_last_group.mul : p.div_group.mul;
    d.shift = last ? p.div_last_group.shift : p.div_group.shift;
    tn = (int)fast_div((u32)in_g, d);
    tm = first + in_g - tn * gsz;
}

// fold: z (+)= sum_s sext(P_s) << 8s for the wave's 32 x 32 sub-tile, which is 2 x 2 blocks of 16 x 16; lane i
// holds rows 4*(i/16) .. +3 of column i%16 of each block.  P_4..P_7 only reach bits 32..63.  Modes: plain store
// (one fold, one split), read-add-write by the owning lane (later folds of a single split), atomic add into a
// zero-filled z (split-K: integer sums mod 2^64 are exact in any order).  The lane index passes through an empty
// asm so that none of the output addresses or bounds tests can be computed ahead of the K loop, where they would
// sit in registers the loop needs.  REMAP: the rows are scattered over the pixels of a larger tensor (see
// GemmParams::out_*).  ZT: z is stored transposed, [N, M].
template <bool REMAP, bool ZT>
__device__ __forceinline__ void fold_blocks(const GemmParams& p, v4i (&acc)[2][2][8], int row0, int col0, int lane,
                                            bool accumulate) {
    int lane_f = lane;
    asm volatile("" : "+v"(lane_f));
    const int c16 = lane_f & 15, g4 = lane_f >> 4;
    int w8 = 1 << 8, w16 = 1 << 16, w24 = 1 << 24;
    asm volatile("" : "+s"(w8), "+s"(w16), "+s"(w24));
    // MODE 0: plain store, 1: read-add-write, 2: atomic add.  The mode is uniform over the launch: one copy of the
    // element loop per mode instead of two branches per element.
    auto all_elements = [&](auto mode_c) {
        constexpr int MODE = decltype(mode_c)::value;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                const int col = col0 + cb * 16 + c16;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int row = row0 + rb * 16 + 4 * g4 + i;
                    // three signed 32 x 32 -> 64 multiply-adds (the weights 2^8, 2^16, 2^24 sit in scalar registers
                    // the compiler cannot see through: as shifts this is seven 64-bit shifts and adds per element)
                    int64_t lo = (int64_t)acc[rb][cb][0][i];
                    lo += (int64_t)acc[rb][cb][1][i] * (int64_t)w8;
                    lo += (int64_t)acc[rb][cb][2][i] * (int64_t)w16;
                    lo += (int64_t)acc[rb][cb][3][i] * (int64_t)w24;
                    const u32 hi = (u32)acc[rb][cb][4][i] + ((u32)acc[rb][cb][5][i] << 8) +
                                   ((u32)acc[rb][cb][6][i] << 16) + ((u32)acc[rb][cb][7][i] << 24);
                    u64 v = (u64)lo + ((u64)hi << 32);
                    if (row < p.M && col < p.N) {
                        u64 zrow = (u64)row;
                        if constexpr (REMAP) {
                            const u32 b = fast_div((u32)row, p.div_howo);
                            const u32 rem = (u32)row - b * (u32)(p.Ho * p.Wo);
                            const u32 i_ = fast_div(rem, p.div_wo), j_ = rem - i_ * (u32)p.Wo;
                            zrow = ((u64)b * (u64)p.out_H + (u64)(p.out_h0 + p.out_sh * (int)i_)) * (u64)p.out_W +
                                   (u64)(p.out_w0 + p.out_sw * (int)j_);
                        }
                        u64* dst = ZT ? p.z + (u64)col * (u64)p.M + zrow : p.z + zrow * (u64)p.N + (u64)col;
                        if constexpr (MODE == 2) {
                            atomicAdd(reinterpret_cast<unsigned long long*>(dst), (unsigned long long)v);
                        } else {
                            if constexpr (MODE == 1) v += *dst;
                            *dst = v;
                        }
                    }
                }
            }
    };
    if (p.ksplit > 1) all_elements(std::integral_constant<int, 2>{});
    else if (accumulate) all_elements(std::integral_constant<int, 1>{});
    else all_elements(std::integral_constant<int, 0>{});
}

// The digit pairs (l, m), l + m <= 7, of one step in issue order, in two phases.
//   Phase 1: the ten pairs with l >= 4, grouped by m = 0, 1, 2, 3, l descending inside a group (they read
//            digits 4-7 of the left operand, whose single LDS buffer the next slice overwrites in phase 2).
//   Phase 2: the 26 pairs with l <= 3, grouped by m = 2, 3, 0, 1, 4, 5, 6, 7, l descending inside a group.
// A wave keeps four left-operand digits in registers (4-7 in phase 1; digits 3, 2, 1, 0 take the places of
// 7, 6, 5, 4 as those retire) and two right-operand digits (digit m lives in set m & 1 and is fetched when
// the previous holder's group is done; the groups of m = 2, 3 come first in phase 2 because these digits are
// the ones left in registers by phase 1).
struct Pair {
    int l, m;
};
constexpr Pair phase1_pair(int i) {
    int m = 0, cnt = 4;
    while (i >= cnt) { i -= cnt; ++m; --cnt; }
    return Pair{7 - m - i, m};
}
constexpr int phase2_group(int g) { return g < 2 ? g + 2 : (g < 4 ? g - 2 : g); }  // m of the g-th group
constexpr Pair phase2_pair(int i) {
    int g = 0;
    while (true) {
        const int m = phase2_group(g);
        const int cnt = m <= 4 ? 4 : 8 - m;  // digits l = cnt-1 .. 0
        if (i < cnt) return Pair{cnt - 1 - i, m};
        i -= cnt;
        ++g;
    }
}
// first slot after the last MFMA that uses right-operand digit m in its phase
constexpr int phase1_group_end(int m) {
    int slots = 0;
    for (int mm = 0; mm <= m; ++mm) slots += 4 * (4 - mm);
    return slots;
}
constexpr int phase2_group_end(int g) {
    int slots = 0;
    for (int gg = 0; gg <= g; ++gg) {
        const int m = phase2_group(gg);
        slots += 4 * (m <= 4 ? 4 : 8 - m);
    }
    return slots;
}

// ---------------------------------------------------------------------------
// LDS byte offset, inside the slab set of one digit and share, of the unit that thread-slot t (thread id plus a
// multiple of the block size) handles in a tile of `rows` rows: k-group jh, row, 16-byte quarter q.  Row-major
// operands put the four quarters of a 64-byte run on consecutive lanes, transposed ones consecutive rows.
__host__ __device__ constexpr int unit_dst(int t, int rows, bool transposed) {
    const int q = transposed ? (t / rows) & 3 : t & 3;
    const int row = transposed ? t % rows : (t >> 2) % rows;
    const int jh = (t >> 2) / rows;
    return jh * rows * 16 + row * 16 + q * 4;
}
// Distance of unit i from unit 0 of the same thread.  The block size is a multiple of four and either a
// multiple of 4*rows (then row and quarter repeat and only the k-group moves) or a divisor of it whose
// multiples stay inside one k-group per pair of units; both cases make the distance the same for every
// thread, so it is evaluated for thread 0.
__host__ __device__ constexpr int unit_delta(int i, int nt, int rows, bool transposed) {
    return unit_dst(i * nt, rows, transposed) - unit_dst(0, rows, transposed);
}

// A block's range of (tile, slice) units, walked one slice at a time.  Three walkers go over the same
// range at different distances: the MFMA loop, the loads of the left operand one slice ahead of it and
// the loads of the right operand up to two slices ahead.  All members are uniform over the block.
struct Walker {
    int64_t u;          // first unit of the range after the current tile's share of it
    int logical;        // current tile in launch order
    int ks, nk;         // current slice; end of the current tile's slices
};

// STREAM selects the streamed work distribution (see run_index); the classic instantiation has exactly
// one tile per block and compiles to straight-line set-up code.
// The kernel's body takes its parameters as a copy of the kernel argument: the compiler then reads every field once,
// ahead of the loop, instead of fetching fields from the argument buffer inside it (measured on the general patch
// gathers: 20-44 spilled registers become 0-4 and the first layers run 14-20 % faster).
template <class T, int AMODE, int BMODE, bool STREAM>
__device__ __forceinline__ void share_gemm_body(const GemmParams p) {
    constexpr int AU = T::A_UNITS, BU = T::B_UNITS;
    __shared__ __attribute__((aligned(16))) char lds[T::LDS_BYTES];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // The streamed instantiation needs the thread id again whenever it enters a tile, i.e. across the K loop, whose
    // registers are all taken: the wave's number waits in a scalar register and the lane is counted anew (a
    // thread id kept in a vector register was spilled, and its reload at the top of every step came with a wait
    // for ALL outstanding loads).
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    auto thread_id_again = [&]() {
        return wave_u * 64 + (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    };
    const int wm = wave_u % T::WM, wn = wave_u / T::WM;   // uniform over the wave: scalar registers
    const int r16 = lane & 15, kg = lane >> 4;

    // ---- this block's range [u0, u_end) of (tile, slice) units
    const int tiles_m = (p.M + T::BM - 1) / T::BM, tiles_n = (p.N + T::BN - 1) / T::BN;
    const int nb = tiles_m * tiles_n;
    const int nk_all = (int)((p.K + 31) / 32);
    int64_t u0, u_end;
    int logical0 = 0, ks0 = 0;   // classic distribution: the block's tile and first slice, known without a division
    if constexpr (STREAM) {
        const int64_t units = (int64_t)nb * nk_all;
        u0 = (int64_t)run_index((int)gridDim.x) * p.stream_per;
        u_end = u0 + p.stream_per < units ? u0 + p.stream_per : units;
    } else {
        const int run = run_index(nb * p.ksplit);
        const int split = (int)fast_div((u32)run, p.div_tiles), logical = run - split * nb;
        const int per_split = p.per_split;
        const int kb = split * per_split;
        u0 = (int64_t)logical * nk_all + kb;
        u_end = (int64_t)logical * nk_all + (kb + per_split < nk_all ? kb + per_split : nk_all);
        logical0 = logical;
        ks0 = kb;
    }
    if (u0 >= u_end) return;  // uniform over the block

    // take the tile that starts at unit w.u: its slices [w.ks, w.nk)
    auto enter_tile = [&](Walker& w) {
        if constexpr (STREAM) {
            w.logical = (int)(w.u / nk_all);
            w.ks = (int)(w.u - (int64_t)w.logical * nk_all);
        } else {   // one tile per block
            w.logical = logical0;
            w.ks = ks0;
        }
        w.nk = (int64_t)w.ks + (u_end - w.u) < nk_all ? w.ks + (int)(u_end - w.u) : nk_all;
        w.u += w.nk - w.ks;
    };

    constexpr bool A_WIDE = AMODE == A_LINEAR_WIDE, B_WIDEROWS = BMODE == B_WIDE;
    constexpr bool A_LINEAR = AMODE == A_LINEAR_VEC || AMODE == A_LINEAR_SCALAR || A_WIDE;
    constexpr bool A_TR = AMODE == A_TRANS;
    // left-operand modes whose memory is contiguous along m: consecutive lanes take consecutive rows
    constexpr bool A_ROWS = A_TR || AMODE == A_PATCH_T || AMODE == A_CONV_GEN || AMODE == A_CONV_DIL;
    // digit-plane route: both operands arrive split; a thread moves the pieces of one row of each tile
    constexpr bool PLANES = AMODE == A_PLANES || AMODE == A_PLANES_CONV;
    static_assert(PLANES == (BMODE == B_PLANES), "plane operands come in pairs");
    static_assert(!PLANES || (T::NT == 4 * T::BM && T::NT == 8 * T::BN && AU == 2 && BU == 1),
                  "the plane route's piece distribution assumes the 128 x 64 tile");
    // the slices follow the taps of a patch gather (see TapCursor)
    constexpr bool A_TAPS = AMODE == A_CONV_C32 || AMODE == A_PLANES_CONV;
    // right-operand modes whose memory is contiguous along n: consecutive lanes take consecutive rows
    constexpr bool B_TR = BMODE == B_TRANS || BMODE == B_FLIP_C32 || BMODE == B_FLIP_GEN || BMODE == B_PATCH_T;
    // ---- per-thread units.  Row-major operands put the four 16-byte quarters of a
    // 64-byte run on consecutive lanes; transposed operands put consecutive rows there.
    typedef typename std::conditional<AMODE == A_LINEAR_VEC, LinearVec,
            typename std::conditional<AMODE == A_LINEAR_WIDE, LinearWide,
            typename std::conditional<AMODE == A_LINEAR_SCALAR, LinearScalar,
            typename std::conditional<AMODE == A_CONV_C32, ConvC32,
            typename std::conditional<AMODE == A_TRANS, TransScalar,
            typename std::conditional<AMODE == A_PATCH_T, PatchTrans,
            typename std::conditional<AMODE == A_CONV_DIL, ConvDil, ConvGen>::type>::type>::type>::type>::type>::type>::type AGen;
    typedef typename std::conditional<BMODE == B_VEC, LinearVec,
            typename std::conditional<BMODE == B_WIDE, LinearWide,
            typename std::conditional<BMODE == B_SCALAR, LinearScalar,
            typename std::conditional<BMODE == B_FLIP_GEN, FlipGen,
            typename std::conditional<BMODE == B_PATCH_T, PatchTrans, TransScalar>::type>::type>::type>::type>::type BGen;
    PlanesRow pa_row, pb_row;   // plane route: this thread's row of the left and of the right tile
    PlanesPatch pa_patch;
    const u64 w_elems = p.w_elems;
    // view on `elems_total` words starting `base` words in
    auto view = [&](const u64* ptr, u64 elems_total, u64 base) {
        const u64 left = (elems_total - base) * 8u;
        return make_rsrc(ptr + base, left > 0x7FFFFFFFull ? 0x7FFFFFFFu : (u32)left);
    };
    // the same, or an empty view (every offset out of range) when `base` lies past the operand or `ok` is false;
    // written as selects on pointer and size: the views of transposed operands are rebuilt in the K loop, where a
    // branch costs the wave an instruction-fetch bubble
    auto view_if = [&](const u64* ptr, u64 elems_total, u64 base, bool ok) {
        const bool in = ok & (base < elems_total);
        const u64 b = in ? base : 0;
        const u64 left = in ? (elems_total - b) * 8u : 0;
        return make_rsrc(ptr + b, left > 0x7FFFFFFFull ? 0x7FFFFFFFu : (u32)left);
    };

    // ---- loader of the left operand: walker, views rebased per tile so that 32-bit offsets suffice,
    // address generators, tap cursor of the patch gather
    Walker wa_;
    u64 a_base_elems;
    TapCursor tap_a;
    __amdgpu_buffer_rsrc_t rs_xa, rs_xb;
    AGen ag[AU];
    // LDS byte offset of unit 0 inside the slab set of digit 0, first share; where a thread's units go does
    // not depend on the tile, and unit i lies a compile-time distance from unit 0 (see unit_delta)
    // (plane route: row tid % BM, digit tid / BM of the low half; the k-half is the unit)
    const int a_dst0 = PLANES ? (tid % T::BM) * 16 + (tid / T::BM) * T::A_DIG : unit_dst(tid, T::BM, A_ROWS);
    auto setup_a = [&]() {
        // (the thread id passes through an empty asm so that nothing below is computed ahead of the K loop and
        // kept in registers across it: a new tile is entered rarely, the registers are needed all the time)
        int tid_s = tid;
        if constexpr (STREAM) {
            tid_s = thread_id_again();
            asm volatile("" : "+v"(tid_s));
        }
        int tm, tn;
        logical_to_tile(p, tiles_m, tiles_n, wa_.logical, tm, tn);
        const int m0 = tm * T::BM, rows_m = p.M - m0;
        if constexpr (PLANES) {
            const u32 KS = (u32)((AMODE == A_PLANES ? p.K : p.Cin) + 31) >> 5;
            u64 base;   // bytes: the 16-row block of the tile's first row / of its first image's first pixel
            if constexpr (AMODE == A_PLANES) {
                base = (u64)(m0 >> 4) * KS * 4096u;
                pa_row.init(tid_s % T::BM, rows_m, KS, tid_s / T::BM);
            } else {
                base = (((u64)((u32)m0 / (u32)(p.Ho * p.Wo)) * (u64)(p.H * p.W)) >> 4) * KS * 4096u;
                pa_patch.init(p, m0, tid_s % T::BM, rows_m, tid_s / T::BM);
            }
            tap_a.set(p, wa_.ks);
            const u64 left = p.xp_bytes - base;
            const u32 bytes = left > 0x7FFFFFFFull ? 0x7FFFFFFFu : (u32)left;
            rs_xa = make_rsrc(p.xp_a + base, bytes);
            rs_xb = make_rsrc(p.xp_b + base, bytes);
            return;
        }
        if (A_LINEAR) a_base_elems = (u64)m0 * (u64)p.lda;
        else if (A_TR) a_base_elems = (u64)m0;
        else if (AMODE == A_PATCH_T) a_base_elems = 0;
        else a_base_elems = (u64)((u32)m0 / (u32)(p.Ho * p.Wo)) * (u64)p.img_elems;
        tap_a.set(p, wa_.ks);
        rs_xa = view(p.x_a, p.x_elems, a_base_elems);
        rs_xb = view(p.x_b, p.x_elems, a_base_elems);
#pragma unroll
        for (int i = 0; i < AU; ++i) {
            const int t = tid_s + i * T::NT;
            int q = A_ROWS ? (t / T::BM) & 3 : t & 3;
            const int row = A_ROWS ? t % T::BM : (t >> 2) % T::BM;
            int jh = (t >> 2) / T::BM;
            // one wave's lanes share the quarter and the k-group when they take consecutive rows: said so, the
            // arithmetic on a unit's k indices (bounds, pixel decomposition) runs on the scalar unit
            if constexpr (A_ROWS && T::BM % 64 == 0) {
                q = __builtin_amdgcn_readfirstlane(q);
                jh = __builtin_amdgcn_readfirstlane(jh);
            }
            ag[i].init(p, m0, row, rows_m, A_TR ? (u32)p.M : (u32)p.lda, q, jh);
        }
    };
    // ---- loader of the right operand
    Walker wb_;
    u64 b_base_elems;
    TapCursor tap_b;   // B_FLIP_C32 and the slice order of the patch gather follow the left operand's taps
    __amdgpu_buffer_rsrc_t rs_wa, rs_wb;
    BGen bg[BU];
    const int b_dst0 = PLANES ? (tid % T::BN) * 16 + (tid / T::BN) * T::B_DIG : unit_dst(tid, T::BN, B_TR);
    auto setup_b = [&]() {
        int tid_s = tid;
        if constexpr (STREAM) {
            tid_s = thread_id_again();
            asm volatile("" : "+v"(tid_s));
        }
        int tm, tn;
        logical_to_tile(p, tiles_m, tiles_n, wb_.logical, tm, tn);
        const int n0 = tn * T::BN, rows_n = p.N - n0;
        if constexpr (PLANES) {
            const u32 KS = (u32)(p.K + 31) >> 5;
            const u64 base = (u64)(n0 >> 4) * KS * 4096u;
            pb_row.init(tid_s % T::BN, rows_n, KS, tid_s / T::BN);
            tap_b.set(p, wb_.ks);
            const u64 left = p.wp_bytes - base;
            const u32 bytes = left > 0x7FFFFFFFull ? 0x7FFFFFFFu : (u32)left;
            rs_wa = make_rsrc(p.wp_a + base, bytes);
            rs_wb = make_rsrc(p.wp_sum + base, bytes);   // the registers of w_b hold w_a + w_b on this route
            return;
        }
        b_base_elems = BMODE == B_PATCH_T ? 0 : (B_TR ? (u64)n0 : (u64)n0 * (u64)p.K);
        tap_b.set(p, wb_.ks);
        rs_wa = view(p.w_a, w_elems, b_base_elems);
        rs_wb = view(p.w_b, w_elems, b_base_elems);
#pragma unroll
        for (int i = 0; i < BU; ++i) {
            const int t = tid_s + i * T::NT;
            int q = B_TR ? (t / T::BN) & 3 : t & 3;
            const int row = B_TR ? t % T::BN : (t >> 2) % T::BN;
            int jh = (t >> 2) / T::BN;
            if constexpr (B_TR && T::BN % 64 == 0) {  // see the left operand
                q = __builtin_amdgcn_readfirstlane(q);
                jh = __builtin_amdgcn_readfirstlane(jh);
            }
            // pitch between consecutive k of one row: N for a transposed matrix, one output
            // channel of the filter (kh*kw*N words) for the flipped filter
            const u32 pitch = BMODE == B_FLIP_C32 ? (u32)(p.flt_kh * p.flt_kw) * (u32)p.N : (B_TR ? (u32)p.N : (u32)p.K);
            bg[i].init(p, n0, row, rows_n, pitch, q, jh);
        }
    };
    // next slice of a loader: the next tile of the range when the current one is used up (streamed
    // distribution only); past the end of the range the slice index just runs on, and what is loaded
    // there (zeros beyond K, or words of the next K range) is never used
    auto advance = [&](Walker& w, auto&& setup) {
        ++w.ks;
        if constexpr (STREAM) {
            if (w.ks == w.nk && w.u < u_end) {  // uniform
                enter_tile(w);
                setup();
            }
        }
    };
    wa_.u = u0;
    enter_tile(wa_);
    setup_a();
    wb_ = wa_;
    setup_b();

    // transposed operands: one view per K slice
    auto a_view = [&](const u64* ptr, __amdgpu_buffer_rsrc_t fixed, int ks) {
        if constexpr (A_TR) {
            const u64 base = a_base_elems + (u64)ks * 32u * (u64)p.M;
            return view_if(ptr, p.x_elems, base, true);
        } else if constexpr (AMODE == A_PATCH_T) {
            const u64 base = (u64)fast_div(32u * (u32)ks, p.div_howo) * p.img_elems;
            return view_if(ptr, p.x_elems, base, true);
        } else {
            return fixed;
        }
    };
    // (B_FLIP_C32 reads the right operand's tap cursor, which load_w moves to slice ks first)
    auto b_view = [&](const u64* ptr, __amdgpu_buffer_rsrc_t fixed, int ks) {
        if constexpr (BMODE == B_TRANS) {
            const u64 base = b_base_elems + (u64)ks * 32u * (u64)p.N;
            return view_if(ptr, w_elems, base, true);
        } else if constexpr (BMODE == B_FLIP_C32) {
            const int ftap = (p.flt_r0 + p.flt_sh * (p.kh - 1 - tap_b.r)) * p.flt_kw + p.flt_s0 + p.flt_sw * (p.kw - 1 - tap_b.s);
            const u64 base = b_base_elems + ((u64)tap_b.c0 * (u64)(p.flt_kh * p.flt_kw) + (u64)ftap) * (u64)p.N;
            return view_if(ptr, w_elems, base, tap_b.c0 < p.Cin);   // (c0 >= Cin: past the end of K)
        } else if constexpr (BMODE == B_PATCH_T) {
            const u64 base = (u64)fast_div(32u * (u32)ks, p.div_howo) * p.img_elems;
            return view_if(ptr, w_elems, base, true);
        } else {
            return fixed;
        }
    };

    // Staging registers: the raw words of one slice of the four share tensors.  They are filled in three
    // batches (first share of the left operand, second share, right operand), each about a third of a step
    // ahead of its split, so that only two batches are ever alive at one time.
    u4 xa[AU][2], xb[AU][2], wa[BU][2], wb[BU][2];

    auto load_a = [&](__amdgpu_buffer_rsrc_t rs, int ks, u4 (*dst)[2]) {
        if constexpr (PLANES) {
            // unit g = k-half: its low-digit piece (cq) and its high-digit piece (cq + 4)
            u32 off;
            if constexpr (AMODE == A_PLANES) {
                off = pa_row.off0 + (u32)ks * 4096u;
            } else {
                tap_a.advance_to(p, ks);
                off = pa_patch.offset(p, tap_a);
            }
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                dst[g][0] = __builtin_amdgcn_raw_buffer_load_b128(rs, off + 2048u * g, 0, 0);
                dst[g][1] = __builtin_amdgcn_raw_buffer_load_b128(rs, off + 2048u * g + 1024u, 0, 0);
            }
        } else if constexpr (AMODE == A_CONV_C32) {
            tap_a.advance_to(p, ks);
#pragma unroll
            for (int i = 0; i < AU; ++i) ag[i].load(p, rs, tap_a, dst[i]);
        } else if constexpr (A_WIDE) {
            (void)rs;   // see load_xa / load_xb
        } else {
#pragma unroll
            for (int i = 0; i < AU; ++i) ag[i].load(p, rs, ks, (u32)p.K, dst[i]);
        }
    };
    // A loader that has run past the last slice of the block's range loads through empty views: every offset is
    // out of range there, so the loads return zeros without touching memory (no branch around them: a branch
    // would make the compiler wait for all outstanding loads where the paths join).
    auto dead_view = [&](__amdgpu_buffer_rsrc_t r, const u64* ptr, bool live) { return live ? r : make_rsrc(ptr, 0); };
    // (long rows: plain pointers instead of views, null past the range)
    auto load_a_wide = [&](const u64* ptr, u4 (*dst)[2]) {
        if constexpr (A_WIDE) {
            const u64* tile = wa_.ks < wa_.nk ? ptr + a_base_elems : nullptr;
#pragma unroll
            for (int i = 0; i < AU; ++i) ag[i].load_wide(tile, wa_.ks, (u32)p.K, dst[i]);
        }
    };
    auto load_xa = [&]() {
        if constexpr (A_WIDE) load_a_wide(p.x_a, xa);
        else load_a(dead_view(a_view(p.x_a, rs_xa, wa_.ks), p.x_a, wa_.ks < wa_.nk), wa_.ks, xa);
    };
    auto load_xb = [&]() {
        if constexpr (A_WIDE) load_a_wide(p.x_b, xb);
        else load_a(dead_view(a_view(p.x_b, rs_xb, wa_.ks), p.x_b, wa_.ks < wa_.nk), wa_.ks, xb);
    };
    auto load_w = [&]() {
        const int ks = wb_.ks;
        int kb = ks;
        if constexpr (A_TAPS) {  // the right operand follows the left operand's slice order (see TapCursor)
            tap_b.advance_to(p, ks);
            kb = tap_b.pks(p);
        }
        const bool live = ks < wb_.nk;
        const __amdgpu_buffer_rsrc_t ra = dead_view(b_view(p.w_a, rs_wa, ks), p.w_a, live),
                                     rb = dead_view(b_view(p.w_b, rs_wb, ks), p.w_b, live);
        if constexpr (PLANES) {
            // digit cq of both k-halves, from the planes of w_a and of w_a + w_b
            const u32 off = pb_row.off0 + (u32)kb * 4096u;
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                wa[0][g] = __builtin_amdgcn_raw_buffer_load_b128(ra, off + 2048u * g, 0, 0);
                wb[0][g] = __builtin_amdgcn_raw_buffer_load_b128(rb, off + 2048u * g, 0, 0);
            }
        } else if constexpr (B_WIDEROWS) {
            (void)ra; (void)rb;
            const u64 *ta = live ? p.w_a + b_base_elems : nullptr, *tb = live ? p.w_b + b_base_elems : nullptr;
#pragma unroll
            for (int i = 0; i < BU; ++i) bg[i].load_wide(ta, kb, (u32)p.K, wa[i]);
#pragma unroll
            for (int i = 0; i < BU; ++i) bg[i].load_wide(tb, kb, (u32)p.K, wb[i]);
        } else {
#pragma unroll
            for (int i = 0; i < BU; ++i) bg[i].load(p, ra, kb, (u32)p.K, wa[i]);
#pragma unroll
            for (int i = 0; i < BU; ++i) bg[i].load(p, rb, kb, (u32)p.K, wb[i]);
        }
    };

    // The split of one unit in four pieces, so that they can be placed between MFMAs:
    // 0: recode the first two words, 1: the last two, 2: digits 0-3 to LDS, 3: digits 4-7.
    // `add` (the first share of the right operand) is summed in before recoding.
    auto unit_op = [&](u4 (&v)[2], const u4 (*add)[2], char* lo, char* hi, auto dig_c, auto phase_c) {
        constexpr int DIG = decltype(dig_c)::value, phase = decltype(phase_c)::value;
        if constexpr (phase < 2) {
            if (add) v[phase] = add64x2(v[phase], (*add)[phase]);
            recode2(v[phase]);
        } else {
            u32 d[4];
            if constexpr (phase == 2) transpose4(v[0].x, v[0].z, v[1].x, v[1].z, d);
            else transpose4(v[0].y, v[0].w, v[1].y, v[1].w, d);
            char* dst = phase == 2 ? lo : hi;
#pragma unroll
            for (int l = 0; l < 4; ++l) *reinterpret_cast<u32*>(dst + l * DIG) = d[l];
        }
    };
    // Pieces of the three batches.  Right operand: the units of w_a + w_b (formed in the registers of w_b,
    // which must happen before w_a is recoded in place), then those of w_a.
    constexpr int NOPS_X = 4 * AU, NOPS_W = 8 * BU;
    // a_lo / a_hi / b_all: LDS byte addresses of this thread's unit 0 in the buffers written (digit 0, first share)
    auto split_x = [&](auto op_c, u4 (*x)[2], auto share_c, int a_lo, int a_hi) {
        constexpr int op = decltype(op_c)::value, unit = op / 4;
        if constexpr (PLANES) {   // the pieces are stored as they are: the low-digit one, then the high-digit one
            constexpr int poff = decltype(share_c)::value * 2 * T::A_RS + unit * T::A_RS;
            if constexpr (op % 4 == 2) *reinterpret_cast<u4*>(lds + a_lo + poff) = x[unit][0];
            if constexpr (op % 4 == 3) *reinterpret_cast<u4*>(lds + a_hi + poff) = x[unit][1];
            return;
        }
        constexpr int off = decltype(share_c)::value * 2 * T::A_RS + unit_delta(unit, T::NT, T::BM, A_ROWS);
        unit_op(x[unit], nullptr, lds + a_lo + off, lds + a_hi + off, std::integral_constant<int, T::A_DIG>{},
                std::integral_constant<int, op % 4>{});
    };
    auto split_w = [&](auto op_c, int b_all) {
        constexpr int op = decltype(op_c)::value, unit = op / 4;
        if constexpr (PLANES) {   // unit 0: pieces of w_a + w_b (k-groups 0, 1); unit 1: pieces of w_a (k-groups 2, 3)
            if constexpr (op % 4 >= 2) {
                constexpr int g = op % 4 - 2;
                *reinterpret_cast<u4*>(lds + b_all + (2 * unit + g) * T::B_RS) = unit == 0 ? wb[0][g] : wa[0][g];
            }
            return;
        }
        const std::integral_constant<int, T::B_DIG> bdig;
        const std::integral_constant<int, op % 4> phase;
        if constexpr (unit < BU) {
            constexpr int off = unit_delta(unit, T::NT, T::BN, B_TR);
            unit_op(wb[unit], &wa[unit], lds + b_all + off, lds + b_all + 4 * T::B_DIG + off, bdig, phase);
        } else {
            constexpr int off = 2 * T::B_RS + unit_delta(unit - BU, T::NT, T::BN, B_TR);
            unit_op(wa[unit - BU], nullptr, lds + b_all + off, lds + b_all + 4 * T::B_DIG + off, bdig, phase);
        }
    };
    // A byte address in LDS kept in a register of its own: every access then is this register plus a 16-bit
    // immediate.  (Left to itself the compiler folds all addresses onto one base and spends an instruction
    // per access on offsets beyond the immediate's range.)
    auto pin = [](int v) {
        asm volatile("" : "+v"(v));
        return v;
    };

    // fragment addresses of this lane: row r16 of a 16-row block, k-group kg
    const int a_frag = kg * T::A_RS + (wm * 32 + r16) * 16;
    const int b_frag = kg * T::B_RS + (wn * 32 + r16) * 16;
    const int a_hi_rd = pin(T::OFF_AHI + a_frag);   // the two addresses that do not change from step to step
    const int a_hi_wr = pin(T::OFF_AHI + a_dst0);

    v4i acc[2][2][8];
    v4i af[4][2], bf[2][2];  // four digits of the left operand, two of the right one; two 16-row blocks each

    // One step: the 144 MFMAs of a slice with a hand-placed issue order (every index is a compile-time
    // constant, a full scheduling fence after every slot keeps the compiler from regrouping them).
    // Buffers `par` hold this step's slice (digits 0-3 of the left operand, all digits of the right one), the
    // other buffers receive the next slice; digits 4-7 of the left operand have one buffer, read in phase 1 and
    // rewritten in phase 2, hence the barrier between them.
    // Between the MFMAs the next slice is prepared, spread evenly over the step (slots counted over both
    // phases): the right operand's words, loaded late in the step before, are split in slots W0..W1; the
    // left operand's first share is loaded at XA_LOAD and split in XA0..XA1 (its digits 4-7 can only be
    // written in phase 2), the second share at XB_LOAD (into the registers the right operand has left) and
    // split in XB0..XB1; W_LOAD then fetches the right operand of the slice after the next.
    constexpr int N1 = 40, N2 = 104;
    constexpr int W0 = 3, W1 = 39, XA_LOAD = 1, XA0 = 42, XA1 = 92, XB_LOAD = 41, XB0 = 94, XB1 = 142, W_LOAD = 93;
    // LIVE = false is the step that computes the last slice of the block's range: nothing is left to prepare.
    auto step = [&](int par, auto live_c) {
        constexpr bool LIVE = decltype(live_c)::value;
        const int a_lo_rd = pin(par * T::A_HALF + a_frag), b_rd = pin(T::OFF_B + par * T::B_ALL + b_frag);
        const int a_lo_wr = pin((par ^ 1) * T::A_HALF + a_dst0), b_wr = pin(T::OFF_B + (par ^ 1) * T::B_ALL + b_dst0);
        auto read_a_hi = [&](int l) {   // digit l in 4..7 -> register set l - 4
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
                af[l - 4][rb] = *reinterpret_cast<const v4i*>(lds + a_hi_rd + (l - 4) * T::A_DIG + rb * 256);
        };
        auto read_a_lo = [&](int l) {   // digit l in 0..3 -> register set l
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
                af[l][rb] = *reinterpret_cast<const v4i*>(lds + a_lo_rd + l * T::A_DIG + rb * 256);
        };
        auto read_b = [&](int m) {      // digit m -> register set m & 1
#pragma unroll
            for (int cb = 0; cb < 2; ++cb)
                bf[m & 1][cb] = *reinterpret_cast<const v4i*>(lds + b_rd + m * T::B_DIG + cb * 256);
        };
        // what goes between the MFMAs of slot `slot` (0..143 over both phases)
        auto between = [&](auto slot_c) {
            constexpr int slot = decltype(slot_c)::value;
            if constexpr (!LIVE) return;
            if constexpr (slot == XA_LOAD) load_xa();
            if constexpr (slot == XB_LOAD) load_xb();
            if constexpr (slot == W_LOAD) load_w();
            if constexpr (slot >= W0 && slot < W1) {
                constexpr int lo = (slot - W0) * NOPS_W / (W1 - W0), hi = (slot - W0 + 1) * NOPS_W / (W1 - W0);
                static_for<lo, hi>([&](auto op_c) { split_w(op_c, b_wr); });
            }
            if constexpr (slot >= XA0 && slot < XA1) {
                constexpr int lo = (slot - XA0) * NOPS_X / (XA1 - XA0), hi = (slot - XA0 + 1) * NOPS_X / (XA1 - XA0);
                static_for<lo, hi>([&](auto op_c) { split_x(op_c, xa, std::integral_constant<int, 0>{}, a_lo_wr, a_hi_wr); });
            }
            if constexpr (slot >= XB0 && slot < XB1) {
                constexpr int lo = (slot - XB0) * NOPS_X / (XB1 - XB0), hi = (slot - XB0 + 1) * NOPS_X / (XB1 - XB0);
                static_for<lo, hi>([&](auto op_c) { split_x(op_c, xb, std::integral_constant<int, 1>{}, a_lo_wr, a_hi_wr); });
            }
        };
        // ---- phase 1: fragments in the order of first use; only the first pair's are awaited before the first MFMA
        read_a_hi(7); read_b(0);
        read_a_hi(6); read_a_hi(5); read_a_hi(4); read_b(1);
        __builtin_amdgcn_sched_barrier(0);
        static_for<0, N1>([&](auto slot_c) {
            constexpr int slot = decltype(slot_c)::value;
            constexpr Pair pr = phase1_pair(slot / 4);
            constexpr int rb = (slot >> 1) & 1, cb = slot & 1;
            acc[rb][cb][pr.l + pr.m] = __builtin_amdgcn_mfma_i32_16x16x64_i8(
                af[pr.l - 4][rb], bf[pr.m & 1][cb], acc[rb][cb][pr.l + pr.m], 0, 0, 0);
            if constexpr (slot + 1 == phase1_group_end(0)) read_b(2);
            if constexpr (slot + 1 == phase1_group_end(1)) read_b(3);
            // a retired high digit hands its registers to a low digit of the same slice (already in LDS):
            // digit 7 is last used by pair 0, digit 6 by pair 4, digit 5 by pair 7
            if constexpr (slot == 3) read_a_lo(3);
            else if constexpr (slot == 19) read_a_lo(2);
            else if constexpr (slot == 31) read_a_lo(1);
            between(slot_c);
            __builtin_amdgcn_sched_barrier(0);
        });
        __syncthreads();   // every wave has read digits 4-7: their buffer may be rewritten
        read_a_lo(0);
        __builtin_amdgcn_sched_barrier(0);
        static_for<0, N2>([&](auto slot_c) {
            constexpr int slot = decltype(slot_c)::value;
            constexpr Pair pr = phase2_pair(slot / 4);
            constexpr int rb = (slot >> 1) & 1, cb = slot & 1;
            acc[rb][cb][pr.l + pr.m] = __builtin_amdgcn_mfma_i32_16x16x64_i8(
                af[pr.l][rb], bf[pr.m & 1][cb], acc[rb][cb][pr.l + pr.m], 0, 0, 0);
            // when the g-th group is done its digit's registers take the digit of group g + 2
            static_for<0, 6>([&](auto g_c) {
                constexpr int g = decltype(g_c)::value;
                if constexpr (slot + 1 == phase2_group_end(g)) read_b(phase2_group(g + 2));
            });
            between(std::integral_constant<int, N1 + slot>{});
            __builtin_amdgcn_sched_barrier(0);
        });
        __syncthreads();   // the next slice is in LDS
    };

    auto clear_acc = [&]() {
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                for (int s = 0; s < 8; ++s) acc[rb][cb][s] = v4i{0, 0, 0, 0};
    };

    // Prologue: the first slice goes to buffer 0 and the right operand of the second slice is requested.
    // Loads past the end of K are out of range and return zeros that are never used, so the loop body
    // needs no "is there a next slice" branch.
    load_xa();
    load_xb();
    advance(wa_, setup_a);
    load_w();
    advance(wb_, setup_b);
    static_for<0, NOPS_X>([&](auto op_c) { split_x(op_c, xa, std::integral_constant<int, 0>{}, a_dst0, a_hi_wr); });
    static_for<0, NOPS_X>([&](auto op_c) { split_x(op_c, xb, std::integral_constant<int, 1>{}, a_dst0, a_hi_wr); });
    static_for<0, NOPS_W>([&](auto op_c) { split_w(op_c, T::OFF_B + b_dst0); });
    load_w();
    advance(wb_, setup_b);
    __syncthreads();
    int par = 0;   // buffer holding the current slice

    // One pass of the outer loop per tile.  In the streamed scheme the loaders run straight on into the
    // next tile of the range, so that only the fold separates two tiles.
    Walker wc;
    wc.u = u0;
    while (true) {
        enter_tile(wc);
        int tm, tn;
        logical_to_tile(p, tiles_m, tiles_n, wc.logical, tm, tn);
        const int fm0 = tm * T::BM + wm * 32, fn0 = tn * T::BN + wn * 32;   // the wave's sub-tile
        const bool ends_here = !STREAM || wc.u >= u_end;   // the block's range ends with this tile
        // one pass per segment of at most SEG_KSTEPS slices (a single pass unless K > 32*SEG_KSTEPS)
        for (int ks0 = wc.ks; ks0 < wc.nk; ks0 += SEG_KSTEPS) {
            const int ke = ks0 + SEG_KSTEPS < wc.nk ? ks0 + SEG_KSTEPS : wc.nk;
            // the very last slice of the range runs outside the loop, in a step that prepares nothing (classic
            // distribution only: its blocks are short; the streamed kernel's long ranges gain little from it and
            // the second copy of the step costs its loop registers)
            const bool final_seg = !STREAM && ends_here && ke == wc.nk;
            const int ke_live = final_seg ? ke - 1 : ke;
            clear_acc();
            for (int ks = ks0; ks < ke_live; ++ks) {
                step(par, std::true_type{});
                // the loaders move on between two steps, where no fragment registers are alive (entering a
                // new tile computes many addresses)
                advance(wa_, setup_a);
                advance(wb_, setup_b);
                par ^= 1;
            }
            if (final_seg) {
                step(par, std::false_type{});
                par ^= 1;
            }
            fold_blocks<BMODE == B_FLIP_C32, AMODE == A_PATCH_T>(p, acc, fm0, fn0, STREAM ? thread_id_again() & 63 : lane,
                                                                 ks0 > wc.ks || p.z_add != 0);
        }
        if (!STREAM || wc.u >= u_end) break;
    }
}

template <class T, int AMODE, int BMODE, bool STREAM>
__global__ __launch_bounds__(T::NT, 1) void share_gemm_kernel(const GemmParams p) {
    share_gemm_body<T, AMODE, BMODE, STREAM>(p);
}

// ===========================================================================
// Digit-plane route.  The split of a word into digits is the same whoever uses
// the word, yet a tile of the left operand is needed by every block column and,
// in a convolution, by every filter tap.  With caller-supplied scratch memory
// the split is therefore done ONCE per operand by to_planes_kernel, which writes
// the digits as int8 "planes", and the product kernel (address modes A_PLANES,
// A_PLANES_CONV, B_PLANES) only moves 16-byte pieces from memory to LDS: no
// vector-ALU work per MFMA.
//
// Plane format of a row-major [R, K] operand, KS = ceil(K/32) slices per row, rows in
// blocks of 16:
//     byte (row, ks, c, j) at (((row/16)*KS + ks)*16 + c)*256 + (row%16)*16 + j,  c = 8*g + l,
// holds digit l of word k = 32*ks + 16*g + j (zero beyond K and beyond R): a piece of 16
// bytes is one MFMA operand register set for one k-half g, and the sixteen rows of a
// block lie next to each other piece by piece, which is the order the product kernel's
// LDS planes have.  The format has the size of the raw operand (rows padded to a
// multiple of 16, K to whole slices).
// ===========================================================================

#if CG_G0
// One thread converts four consecutive words of a row; the 64 lanes of a wave take the four
// 4-word quarters of one k-half of sixteen rows, so that each of their eight stores (one per
// digit) writes 256 contiguous bytes.  One launch converts all four tensors of a product:
// a block takes the job its index falls into.
struct PlaneJob {
    const u64 *src, *add;   // add: summed in before the split (w_a + w_b), or null
    char* dst;
    u32 R, K, KS;
    u32 first_block;        // blocks [first_block, next job's first_block) work on this job
};
struct PlaneJobs {
    PlaneJob job[4];
    u32 total_blocks;
};

__global__ __launch_bounds__(256) void to_planes_kernel(const PlaneJobs jobs) {
    int ji = 0;
#pragma unroll
    for (int i = 1; i < 4; ++i)
        if (blockIdx.x >= jobs.job[i].first_block) ji = i;
    const PlaneJob& jb = jobs.job[ji];
    const u32 end_block = ji < 3 ? jobs.job[ji + 1].first_block : jobs.total_blocks;
    const u64 nblocks = end_block - jb.first_block;
    const u32 R = jb.R, K = jb.K, KS = jb.KS;
    const u64 rb_count = (R + 15) / 16;
    const u64 units = rb_count * KS * 2 * 64;  // per row block, slice and k-half: 16 rows x 4 quarters
    for (u64 ui = (u64)(blockIdx.x - jb.first_block) * 256 + threadIdx.x; ui < units; ui += nblocks * 256) {
        const u32 lane = (u32)(ui & 63), q = lane & 3, r16 = lane >> 2;
        const u64 grp = ui >> 6;
        const u32 g = (u32)(grp & 1);
        const u64 bs = grp >> 1;                 // (row block, slice)
        const u32 ks = (u32)(bs % KS);
        const u64 rb = bs / KS;
        const u64 row = rb * 16 + r16;
        const u32 k0 = 32 * ks + 16 * g + 4 * q;  // first word of the unit
        u4 v0 = {0, 0, 0, 0}, v1 = {0, 0, 0, 0};
        if (row < R) {
            const u64* s_ = jb.src + row * K + k0;
            const u64* a = jb.add ? jb.add + row * K + k0 : nullptr;
            if (k0 < K) {  // K is even: words come in valid pairs
                v0 = *reinterpret_cast<const u4*>(s_);
                if (a) v0 = add64x2(v0, *reinterpret_cast<const u4*>(a));
            }
            if (k0 + 2 < K) {
                v1 = *reinterpret_cast<const u4*>(s_ + 2);
                if (a) v1 = add64x2(v1, *reinterpret_cast<const u4*>(a + 2));
            }
        }
        recode2(v0);
        recode2(v1);
        u32 d[8];
        transpose4(v0.x, v0.z, v1.x, v1.z, d);
        transpose4(v0.y, v0.w, v1.y, v1.w, d + 4);
        char* o = jb.dst + ((bs * 16 + 8 * g) * 256) + r16 * 16 + q * 4;
#pragma unroll
        for (int l = 0; l < 8; ++l) *reinterpret_cast<u32*>(o + l * 256) = d[l];
    }
}

// z = 0 ahead of a split-K launch (a kernel, not a memset, so that callers may
// capture the stream into a graph)
__global__ __launch_bounds__(256) void zero_fill_kernel(u64* z, size_t n) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) z[i] = 0;
}

#endif  // CG_G0

template <class T, int AMODE, int BMODE>
static hipError_t launch(const GemmParams& p, hipStream_t stream);

// Blocks that run at one time: a block's LDS leaves room for one block per compute unit.
static constexpr int ROUND_BLOCKS = 256;
// A K range of a split holds at least this many slices.
static constexpr int SPLIT_MIN_SLICES = 2;
// Cost of the fixed part of a block (prologue, fold of the accumulators into z), in
// units of one K slice of the main loop, with a plain store and with atomic adds.
static constexpr double SPLIT_COST_PLAIN = 1.0, SPLIT_COST_ATOMIC = 2.0;
// The streamed distribution must beat the classic one by this factor of modelled time to be used.
static constexpr double STREAM_MARGIN = 0.88;
// Several rounds of unsplit tiles of at most this many slices are run as one round of blocks that
// each walk through whole tiles.
static constexpr int PERSIST_MAX_SLICES = 32;

static int choose_ksplit(int64_t tiles, int nk) {
    // A block's 160 KB of LDS leaves room for one block per compute unit, so a grid runs
    // in rounds of 256 blocks and the last round costs as much as a full one.  Splitting
    // K makes the blocks shorter, which fills the chip when the tiles alone cannot and
    // shrinks the idle part of the last round otherwise.  The split count with the least
    // modelled time wins: rounds * (slices per block + fixed cost per block).
    const int units = ROUND_BLOCKS;
    int64_t max_split = 8 * units / tiles;  // at most eight rounds' worth of blocks
    if (max_split > nk / SPLIT_MIN_SLICES) max_split = nk / SPLIT_MIN_SLICES;
    int best = 1;
    double best_cost = 0;
    for (int64_t ks = 1; ks <= (max_split < 1 ? 1 : max_split); ++ks) {
        const int64_t per = (nk + ks - 1) / ks;
        const int64_t eff = (nk + per - 1) / per;  // no empty splits
        if (eff != ks) continue;
        const int64_t rounds = (tiles * eff + units - 1) / units;
        const double cost = (double)rounds * ((double)per + (eff > 1 ? SPLIT_COST_ATOMIC : SPLIT_COST_PLAIN));
        if (ks == 1 || cost < best_cost * 0.97) {  // a split must pay for itself by a margin
            best = (int)eff;
            best_cost = cost;
        }
    }
    return best;
}

// Tile-rows per launch-order group.  An XCD's run of `run` consecutive tiles covers
// rows x cols tiles and fetches that many tile-rows of the left operand's tensor and
// tile-columns of the right operand's (of the split's K range); the group height that
// minimises the bytes wins (ties go to the smaller group, which keeps the tiles that
// run at the same time closer together).  For a convolution the left tensor is the
// image, not the (kh*kw times larger) patch matrix: the taps of a tile hit in L2.
//
// Two row-major matrices (matmul, either route) do not follow the byte count: measured on products of 1024 to
// 16384 rows and columns, K = 1024 .. 8192, the best group is 2 tile-rows when the left operand has 32 tile-rows
// or more and 4 below that, whatever the byte count prefers (8 and 16 for 4096^3 and 8192 x 8192 x 2048, which
// run 3 % and 10 % slower that way: the left operand's slices are requested one step ahead of their use, the
// right operand's two, so a miss on the left operand is the one that stalls a block, and a low group lets sixteen
// blocks of an XCD share each slice of it).  When a block walks through whole tiles (`whole_tiles`), tall
// products (four times as many tile-rows as tile columns) run best with the highest group, the others with 2.
static int choose_group_m(const GemmParams& p, int64_t tiles_m, int64_t tiles_n, int ksplit, bool matrix_pair,
                          bool whole_tiles) {
    const double a_row = (double)p.x_elems / (double)tiles_m, b_col = (double)p.w_elems / (double)tiles_n;
    const int64_t nb = tiles_m * tiles_n;
    int64_t run = nb * ksplit / 8;
    if (run < 1) run = 1;
    if (run >= nb) return tiles_n >= 8 ? 4 : (tiles_n >= 2 ? 8 : 32);  // whole splits per XCD: shape is irrelevant
    if (matrix_pair) {
        if (whole_tiles) return tiles_m >= 4 * tiles_n ? 32 : 2;
        return tiles_m >= 32 ? 2 : 4;
    }
    int best = 1;
    double best_cost = -1;
    for (int64_t g = 1; g <= tiles_m; g *= 2) {
        int64_t rows, cols;
        if (run <= g * tiles_n) {
            rows = run < g ? run : g;
            cols = (run + g - 1) / g;
        } else {
            rows = g * ((run + g * tiles_n - 1) / (g * tiles_n));
            cols = tiles_n;
        }
        const double cost = (double)rows * a_row + (double)cols * b_col;
        if (best_cost < 0 || cost < best_cost) {
            best = (int)g;
            best_cost = cost;
        }
    }
    return best;
}

#if CG_G0
hipError_t launch_zero_words(uint64_t* z, size_t n, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    size_t blocks = (n + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(zero_fill_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, z, n);
    return hipGetLastError();
}
#endif

// z = 0 ahead of a launch whose blocks add into it (unless the caller has done so: a
// scattered output is cleared by the caller, who knows its extent; or z holds a value
// the product is to be added to)
static hipError_t launch_zero_fill(const GemmParams& p, hipStream_t stream) {
    if (p.z_prezeroed || p.z_add) return hipSuccess;
    return launch_zero_words(p.z, (size_t)p.M * (size_t)p.N, stream);
}

#if CG_G0
hipError_t launch_to_planes(const GemmParams& p, int64_t x_rows, int64_t x_k, hipStream_t stream) {
    PlaneJobs jobs;
    const struct { const u64 *src, *add; const char* dst; int64_t R, K; } in[4] = {
        {p.x_a, nullptr, p.xp_a, x_rows, x_k}, {p.x_b, nullptr, p.xp_b, x_rows, x_k},
        {p.w_a, p.w_b, p.wp_sum, p.N, p.K}, {p.w_a, nullptr, p.wp_a, p.N, p.K}};
    u32 first = 0;
    for (int i = 0; i < 4; ++i) {
        const int64_t KS = (in[i].K + 31) / 32;
        const int64_t units = (in[i].R + 15) / 16 * KS * 128;
        int64_t blocks = (units + 255) / 256;
        if (blocks > 256 * 16) blocks = 256 * 16;   // grid stride beyond that
        jobs.job[i] = PlaneJob{in[i].src, in[i].add, const_cast<char*>(in[i].dst), (u32)in[i].R, (u32)in[i].K, (u32)KS, first};
        first += (u32)blocks;
    }
    jobs.total_blocks = first;
    hipLaunchKernelGGL(to_planes_kernel, dim3(first), dim3(256), 0, stream, jobs);
    return hipGetLastError();
}
#endif

// Modelled time of the classic distribution with `ks` splits, in K slices (see choose_ksplit).
static double classic_cost(int64_t tiles, int nk, int ks) {
    const int64_t per = (nk + ks - 1) / ks;
    const int64_t rounds = (tiles * ks + ROUND_BLOCKS - 1) / ROUND_BLOCKS;
    return (double)rounds * ((double)per + (ks > 1 ? SPLIT_COST_ATOMIC : SPLIT_COST_PLAIN));
}

// The streamed distribution is compiled for the address generators of the large layers only.
template <int AMODE, int BMODE>
struct CanStream {
    static constexpr bool value = (AMODE == A_LINEAR_VEC && BMODE == B_VEC) || (AMODE == A_CONV_C32 && BMODE == B_VEC) ||
                                  (AMODE == A_CONV_C32 && BMODE == B_FLIP_C32) || (AMODE == A_TRANS && BMODE == B_PATCH_T) ||
                                  (AMODE == A_PATCH_T && BMODE == B_TRANS);
};

// The weight gradient's classic instantiation spills registers inside the loop (its streamed one does not,
// and is 7 % faster on the same ranges over the VGG-shaped layers): only the streamed one is built.  The input
// gradient keeps both: its unsplit tiles gain more from the classic order's neighbouring tiles per XCD.
template <int AMODE, int BMODE>
struct StreamOnly {
    static constexpr bool value = (AMODE == A_TRANS && BMODE == B_PATCH_T) || (AMODE == A_PATCH_T && BMODE == B_TRANS);
};

template <class T, int AMODE, int BMODE>
static hipError_t launch(const GemmParams& p, hipStream_t stream) {
    const int64_t tiles_m = (p.M + T::BM - 1) / T::BM, tiles_n = (p.N + T::BN - 1) / T::BN;
    const int64_t tiles = tiles_m * tiles_n;
    const int nk = (p.K + 31) / 32;
    GemmParams q = p;
    q.ksplit = choose_ksplit(tiles, nk);
    q.stream_per = 0;
    unsigned grid = (unsigned)(tiles * q.ksplit);
    // Streamed distribution: one block per compute unit, each taking an equal run of (tile, slice)
    // units.  A block pays the fixed cost once per tile its run touches (about per/nk + 1 of them).
    // Worth it when the classic grid leaves a round partly empty.
    const int64_t units = tiles * nk;
    if (CanStream<AMODE, BMODE>::value && units >= 3 * ROUND_BLOCKS && units < ((int64_t)1 << 40)) {
        const int64_t per = (units + ROUND_BLOCKS - 1) / ROUND_BLOCKS;
        const double streamed = (double)per + SPLIT_COST_ATOMIC * ((double)per / nk + 1.0);
        if (streamed < STREAM_MARGIN * classic_cost(tiles, nk, q.ksplit)) {
            q.stream_per = per;
            q.ksplit = 2;  // any value above 1: the folds add atomically into a zero-filled z
            grid = (unsigned)((units + per - 1) / per);
        }
    }
    // Whole tiles streamed: when the classic grid needs several rounds of unsplit tiles with a short K, one
    // block per compute unit walks through an equal run of whole tiles instead.  The kernel's pipeline then
    // runs on from tile to tile (no prologue, no block launch in between) and every tile is still stored
    // plainly.  Measured: 3-9 % on layers of up to 16 slices; with a long K the fixed part of a tile does not
    // matter and the classic order, which keeps the tiles an XCD runs at one time next to each other, is
    // 1-2 % faster.
    // Row-major left operands only: a patch gather re-reads the rows of neighbouring tiles, which hit in L2
    // when the neighbours run at the same time and miss when one block takes them one after the other
    // (measured on the 3x3 layers of the VGG-shaped step: twice the memory reads for 1-3 % of time).
    if (CanStream<AMODE, BMODE>::value && AMODE == A_LINEAR_VEC && q.stream_per == 0 && q.ksplit == 1 &&
        tiles > ROUND_BLOCKS && nk <= PERSIST_MAX_SLICES) {
        const int64_t tiles_per_block = (tiles + ROUND_BLOCKS - 1) / ROUND_BLOCKS;
        q.stream_per = tiles_per_block * nk;
        grid = (unsigned)((tiles + tiles_per_block - 1) / tiles_per_block);
    }
    // The weight gradient runs the streamed kernel also where the classic distribution is the better one: a
    // run of one split's slices is that distribution, tile after tile instead of split after split.
    if (StreamOnly<AMODE, BMODE>::value && q.stream_per == 0) {
        q.stream_per = (nk + q.ksplit - 1) / q.ksplit;
        grid = (unsigned)((units + q.stream_per - 1) / q.stream_per);
    }
    constexpr bool MATRIX_PAIR =
        (AMODE == A_LINEAR_VEC || AMODE == A_LINEAR_SCALAR || AMODE == A_LINEAR_WIDE || AMODE == A_PLANES) &&
        (BMODE == B_VEC || BMODE == B_SCALAR || BMODE == B_WIDE || BMODE == B_PLANES);
    q.group_m = choose_group_m(p, tiles_m, tiles_n, q.stream_per > 0 ? 1 : q.ksplit, MATRIX_PAIR,
                               q.stream_per > 0 && q.ksplit == 1);
    {   // divisors of the blocks' index arithmetic (every divisor is at least 1)
        auto fd = [](int64_t d) { return make_fast_div((uint32_t)(d < 1 ? 1 : d)); };
        q.div_tiles = fd(tiles);
        q.per_split = (nk + q.ksplit - 1) / q.ksplit;
        q.div_per_group = fd((int64_t)q.group_m * tiles_n);
        q.div_group = fd(q.group_m);
        q.div_last_group = fd(tiles_m % q.group_m ? tiles_m % q.group_m : q.group_m);
        q.div_taps = fd((int64_t)q.kh * q.kw);
        q.div_tap_kw = fd(q.kw);
        q.div_row_howo = fd((int64_t)q.Ho * q.Wo);
        q.div_row_wo = fd(q.Wo);
        q.tap_rows = 0;   // bit r*kw for every row r of the tap grid (patch gathers with a tap mask: at most 32 taps)
        if (q.kh >= 1 && q.kw >= 1 && (int64_t)q.kh * q.kw <= 32)
            for (int r = 0; r < q.kh; ++r) q.tap_rows |= 1u << (r * q.kw);
    }
    if (q.ksplit > 1)
        if (hipError_t e = launch_zero_fill(q, stream)) return e;
    if constexpr (CanStream<AMODE, BMODE>::value) {
        if (q.stream_per > 0) {
            hipLaunchKernelGGL((share_gemm_kernel<T, AMODE, BMODE, true>), dim3(grid), dim3(T::NT), 0, stream, q);
            return hipGetLastError();
        }
    }
    if constexpr (!StreamOnly<AMODE, BMODE>::value)
        hipLaunchKernelGGL((share_gemm_kernel<T, AMODE, BMODE, false>), dim3(grid), dim3(T::NT), 0, stream, q);
    return hipGetLastError();
}

// The address-generator pairs of one compiled group; *found says whether (amode, bmode) is one of them.
#define CG_CASE(A, B) if (amode == A && bmode == B) return launch<T, A, B>(p, stream)
#if CG_G0
hipError_t launch_share_gemm_group0(const GemmParams& p, int amode, int bmode, hipStream_t stream, bool* found) {
    typedef DefaultStepTile T;  // 4 waves along M, 2 along N
    *found = true;
    // Fully connected layers at small batch: one 32-row wave tile holds all of M, so a
    // 32 x 128 tile of four waves does a quarter of the matrix work of the 128-row tile
    // (measured: pays from K of a few thousand on; shorter products are launch-bound either way).
    if (amode == A_LINEAR_VEC && bmode == B_VEC && share_gemm_small_applies(p)) return launch_share_gemm_small(p, stream);
    if (amode == A_LINEAR_VEC && bmode == B_VEC && p.M <= 32 && p.N >= 128 && p.K >= 2048)
        return launch<StepTile<1, 4>, A_LINEAR_VEC, B_VEC>(p, stream);
    CG_CASE(A_LINEAR_VEC, B_VEC);
    CG_CASE(A_LINEAR_SCALAR, B_SCALAR);
    CG_CASE(A_PLANES, B_PLANES);
    CG_CASE(A_PLANES_CONV, B_PLANES);
    CG_CASE(A_LINEAR_WIDE, B_WIDE);
    *found = false;
    return hipSuccess;
}
#endif
#if CG_G1
hipError_t launch_share_gemm_group1(const GemmParams& p, int amode, int bmode, hipStream_t stream, bool* found) {
    typedef DefaultStepTile T;
    *found = true;
    CG_CASE(A_CONV_C32, B_VEC);
    CG_CASE(A_CONV_GEN, B_VEC);
    CG_CASE(A_CONV_GEN, B_SCALAR);
    CG_CASE(A_CONV_C32, B_FLIP_C32);
    CG_CASE(A_CONV_GEN, B_FLIP_GEN);
    CG_CASE(A_CONV_DIL, B_FLIP_GEN);
    *found = false;
    return hipSuccess;
}
#endif
#if CG_G2
hipError_t launch_share_gemm_group2(const GemmParams& p, int amode, int bmode, hipStream_t stream, bool* found) {
    typedef DefaultStepTile T;
    *found = true;
    CG_CASE(A_LINEAR_VEC, B_TRANS);
    CG_CASE(A_LINEAR_SCALAR, B_TRANS);
    CG_CASE(A_TRANS, B_VEC);
    CG_CASE(A_TRANS, B_SCALAR);
    CG_CASE(A_TRANS, B_TRANS);
    CG_CASE(A_TRANS, B_PATCH_T);
    CG_CASE(A_PATCH_T, B_TRANS);
    CG_CASE(A_LINEAR_WIDE, B_TRANS);
    CG_CASE(A_TRANS, B_WIDE);
    *found = false;
    return hipSuccess;
}
#endif
#undef CG_CASE

#if CG_G0
hipError_t launch_share_gemm_group1(const GemmParams& p, int amode, int bmode, hipStream_t stream, bool* found);
hipError_t launch_share_gemm_group2(const GemmParams& p, int amode, int bmode, hipStream_t stream, bool* found);

hipError_t launch_share_gemm(const GemmParams& p, int amode, int bmode, hipStream_t stream) {
    bool found = false;
    hipError_t e = launch_share_gemm_group0(p, amode, bmode, stream, &found);
    if (found) return e;
    e = launch_share_gemm_group1(p, amode, bmode, stream, &found);
    if (found) return e;
    e = launch_share_gemm_group2(p, amode, bmode, stream, &found);
    return found ? e : hipErrorInvalidValue;
}
#endif

}  // namespace cg
