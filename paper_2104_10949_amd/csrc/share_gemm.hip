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
// Each 32-wide slice of K therefore yields two "half-steps": an even one
// (x_a against w_a + w_b) and an odd one (x_b against w_a).
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
// |d d'| <= 2^14, and P_s receives (s+1)*32 products per half-step, so P_0..P_3
// stay exact in i32 for 1023 half-steps; P_4..P_7 only matter mod 2^(64-8s) <=
// 2^32, where i32 wraparound (verified on hardware) is harmless.  After at most
// SEG_KSTEPS slices of K the accumulators are folded into the 64-bit result
// z += sum_s sext(P_s) << 8s and cleared.
//
// Data movement.  Each share tile is read from HBM once per block as raw
// uint64 (coalesced 16-byte buffer loads, out-of-range lanes return 0, which
// is exact padding in the ring), split into digit planes in registers
// (4 integer ops + 4 byte permutes per word), written to LDS as
// [digit][k-half][row][16 bytes] so that every MFMA operand is one conflict-free
// ds_read_b128, and consumed by v_mfma_i32_32x32x32_i8.  Convolution uses the
// same kernel: only the address generator of the left operand differs (patch
// gather from NHWC with zero fill).  Nothing but z is written to HBM.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "share_gemm.h"

namespace cg {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));
typedef unsigned int u2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32;
typedef uint64_t u64;

// voffset that is out of range for every buffer view (views are < 2^31 bytes):
// the hardware then returns zeros instead of reading memory.
static constexpr u32 OOB = 0x80000000u;

// Slices of K (32 elements each) between two folds of the i32 accumulators:
// 2*511 = 1022 half-steps <= 1023.
static constexpr int SEG_KSTEPS = 511;

template <int WM_, int WN_, int SM_, int SN_>
struct Tile {
    static constexpr int WM = WM_, WN = WN_, SM = SM_, SN = SN_;
    static constexpr int BM = WM * SM * 32, BN = WN * SN * 32;
    static constexpr int NT = WM * WN * 64;
    // A "unit" is 4 words of one row: two 16-byte loads, one 4x4 byte transpose
    // per 32-bit half, eight 4-byte LDS writes.
    static constexpr int A_UNITS = BM * 8 / NT, B_UNITS = BN * 8 / NT;
    static constexpr int A_RS = BM * 16, B_RS = BN * 16;  // bytes of one [digit][k-half] slab
    static constexpr int A_BYTES = 16 * A_RS, B_BYTES = 16 * B_RS;
    static constexpr int STAGE = A_BYTES + B_BYTES;
    static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile does not divide over the threads");
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, u32 bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

__device__ __forceinline__ u32 fast_div(u32 n, FastDiv d) {
    return ((u32)(((u64)n * d.mul) >> 32) + n) >> d.shift;
}

// signed-digit recoding of one 64-bit word held as (lo, hi)
__device__ __forceinline__ void recode(u32& lo, u32& hi) {
    u64 t = ((u64)hi << 32) | lo;
    t = (t + 0x8080808080808080ull) ^ 0x8080808080808080ull;
    lo = (u32)t;
    hi = (u32)(t >> 32);
}

// 4x4 byte transpose: out[l] = { byte l of a0, byte l of a1, byte l of a2, byte l of a3 }.
// v_perm_b32(S0, S1, sel): selector values 0-3 pick bytes of S1, 4-7 bytes of S0.
__device__ __forceinline__ void transpose4(u32 a0, u32 a1, u32 a2, u32 a3, u32 out[4]) {
    const u32 t0 = __builtin_amdgcn_perm(a1, a0, 0x05010400u);  // a0.b0 a1.b0 a0.b1 a1.b1
    const u32 t1 = __builtin_amdgcn_perm(a1, a0, 0x07030602u);  // a0.b2 a1.b2 a0.b3 a1.b3
    const u32 u0 = __builtin_amdgcn_perm(a3, a2, 0x05010400u);
    const u32 u1 = __builtin_amdgcn_perm(a3, a2, 0x07030602u);
    out[0] = __builtin_amdgcn_perm(u0, t0, 0x05040100u);
    out[1] = __builtin_amdgcn_perm(u0, t0, 0x07060302u);
    out[2] = __builtin_amdgcn_perm(u1, t1, 0x05040100u);
    out[3] = __builtin_amdgcn_perm(u1, t1, 0x07060302u);
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
// ---------------------------------------------------------------------------

// Row-major [rows, ld] operand, 16-byte loads (ld even, base 16-byte aligned).
struct LinearVec {
    u32 rowoff;  // byte offset of the row inside the block's buffer view, or OOB
    u32 kq;      // 16*jh + 2*q
    __device__ __forceinline__ void init(const GemmParams&, int row_local, int rows_left, u32 ld,
                                         int q, int jh) {
        rowoff = row_local < rows_left ? (u32)row_local * ld * 8u : OOB;
        kq = 16 * jh + 2 * q;
    }
    __device__ __forceinline__ void begin_kstep(const GemmParams&, int) {}
    __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, int ks, u32 K, u4 out[2]) const {
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const u32 k = 32u * ks + kq + 8u * jj;
            const u32 off = (k < K && rowoff != OOB) ? rowoff + k * 8u : OOB;
            out[jj] = __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0);
        }
    }
};

// Row-major operand with 8-byte loads: any ld, any 8-byte-aligned base.
struct LinearScalar {
    u32 rowoff;
    u32 kq;
    __device__ __forceinline__ void init(const GemmParams&, int row_local, int rows_left, u32 ld,
                                         int q, int jh) {
        rowoff = row_local < rows_left ? (u32)row_local * ld * 8u : OOB;
        kq = 16 * jh + 2 * q;
    }
    __device__ __forceinline__ void begin_kstep(const GemmParams&, int) {}
    __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, int ks, u32 K, u4 out[2]) const {
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const u32 k = 32u * ks + kq + 8u * jj;
            const u32 o0 = (k < K && rowoff != OOB) ? rowoff + k * 8u : OOB;
            const u32 o1 = (k + 1 < K && rowoff != OOB) ? rowoff + k * 8u + 8u : OOB;
            const u2 e0 = __builtin_amdgcn_raw_buffer_load_b64(r, o0, 0, 0);
            const u2 e1 = __builtin_amdgcn_raw_buffer_load_b64(r, o1, 0, 0);
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
        const u32 b = m / HoWo, b0 = (u32)m0 / HoWo;
        const u32 rem = m - b * HoWo;
        const u32 ho = rem / (u32)p.Wo, wo = rem - ho * (u32)p.Wo;
        hi0 = (int)ho * p.sh - p.ph;
        wi0 = (int)wo * p.sw - p.pw;
        base = (b - b0) * (u32)p.H * (u32)p.W * (u32)p.Cin * 8u +
               ((u32)hi0 * (u32)p.W + (u32)wi0) * (u32)p.Cin * 8u;
    }
};

// Patch gather with Cin % 32 == 0: a 32-word slice of K never straddles a filter
// tap, so the tap (r, s) and the channel offset are uniform over the block.
struct ConvC32 {
    PatchRow pr;
    u32 kq8;       // (16*jh + 2*q) * 8 bytes
    u32 tap_off;   // per k-step: ((r*W + s)*Cin + c0) * 8, block-uniform
    int r, s;
    __device__ __forceinline__ void init(const GemmParams& p, int m0, int row_local, int rows_left,
                                         int q, int jh) {
        pr.init(p, m0, row_local, rows_left);
        kq8 = (16 * jh + 2 * q) * 8;
    }
    __device__ __forceinline__ void begin_kstep(const GemmParams& p, int ks) {
        const u32 k0 = 32u * ks;
        const u32 rs = k0 / (u32)p.Cin;           // uniform: scalar ALU
        const u32 c0 = k0 - rs * (u32)p.Cin;
        r = (int)(rs / (u32)p.kw);
        s = (int)(rs - (u32)r * (u32)p.kw);
        tap_off = (((u32)r * (u32)p.W + (u32)s) * (u32)p.Cin + c0) * 8u;
    }
    __device__ __forceinline__ void load(const GemmParams& p, __amdgpu_buffer_rsrc_t rs_, u4 out[2]) const {
        const bool v = pr.ok && (u32)(pr.hi0 + r) < (u32)p.H && (u32)(pr.wi0 + s) < (u32)p.W;
        const u32 off = pr.base + tap_off + kq8;
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
            out[jj] = __builtin_amdgcn_raw_buffer_load_b128(rs_, v ? off + 64u * jj : OOB, 0, 0);
    }
};

// Patch gather, any Cin: every word finds its own tap.
struct ConvGen {
    PatchRow pr;
    u32 kq;
    __device__ __forceinline__ void init(const GemmParams& p, int m0, int row_local, int rows_left,
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
    __device__ __forceinline__ void load(const GemmParams& p, __amdgpu_buffer_rsrc_t rs_, int ks,
                                         u4 out[2]) const {
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const u32 k = 32u * ks + kq + 8u * jj;
            const u2 e0 = one(p, rs_, k), e1 = one(p, rs_, k + 1);
            out[jj].x = e0.x; out[jj].y = e0.y; out[jj].z = e1.x; out[jj].w = e1.y;
        }
    }
};

// ---------------------------------------------------------------------------
template <class T, int AMODE, bool BVEC>
__global__ __launch_bounds__(T::NT) void share_gemm_kernel(const GemmParams p) {
    constexpr int SM = T::SM, SN = T::SN;
    __shared__ __attribute__((aligned(16))) char lds[2 * T::STAGE];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % T::WM, wn = wave / T::WM;
    const int r32 = lane & 31, h = lane >> 5;

    // ---- block -> output tile.  Consecutive block ids go to different XCDs
    // (round robin over 8), so give each XCD a contiguous run of logical tiles:
    // tiles that share operand rows then share one L2.
    const int tiles_m = (p.M + T::BM - 1) / T::BM, tiles_n = (p.N + T::BN - 1) / T::BN;
    const int nb = tiles_m * tiles_n;
    int logical;
    {
        const int bid = blockIdx.x, xcd = bid & 7, idx = bid >> 3;
        const int per = nb >> 3, rem = nb & 7;
        logical = xcd * per + (xcd < rem ? xcd : rem) + idx;
    }
    // inside the run: groups of GM tile-rows, tile-row fastest inside a group
    int tm, tn;
    {
        const int GM = p.group_m;
        const int per_group = GM * tiles_n;
        const int g = logical / per_group, in_g = logical - g * per_group;
        const int first = g * GM;
        const int gsz = tiles_m - first < GM ? tiles_m - first : GM;
        tm = first + in_g % gsz;
        tn = in_g / gsz;
    }
    const int m0 = tm * T::BM, n0 = tn * T::BN;
    const int rows_m = p.M - m0, rows_n = p.N - n0;

    // ---- buffer views, rebased per block so that 32-bit offsets suffice
    u64 a_base_elems;
    if (AMODE == A_LINEAR_VEC || AMODE == A_LINEAR_SCALAR) a_base_elems = (u64)m0 * (u64)p.lda;
    else a_base_elems = (u64)((u32)m0 / (u32)(p.Ho * p.Wo)) * (u64)p.img_elems;
    const u64 a_left = ((u64)p.x_elems - a_base_elems) * 8u;
    const u32 a_bytes = a_left > 0x7FFFFFFFull ? 0x7FFFFFFFu : (u32)a_left;
    const __amdgpu_buffer_rsrc_t rs_xa = make_rsrc(p.x_a + a_base_elems, a_bytes);
    const __amdgpu_buffer_rsrc_t rs_xb = make_rsrc(p.x_b + a_base_elems, a_bytes);
    const u64 b_base_elems = (u64)n0 * (u64)p.K;
    const u64 b_left = ((u64)p.N * (u64)p.K - b_base_elems) * 8u;
    const u32 b_bytes = b_left > 0x7FFFFFFFull ? 0x7FFFFFFFu : (u32)b_left;
    const __amdgpu_buffer_rsrc_t rs_wa = make_rsrc(p.w_a + b_base_elems, b_bytes);
    const __amdgpu_buffer_rsrc_t rs_wb = make_rsrc(p.w_b + b_base_elems, b_bytes);

    // ---- per-thread units
    typedef typename std::conditional<AMODE == A_LINEAR_VEC, LinearVec,
            typename std::conditional<AMODE == A_LINEAR_SCALAR, LinearScalar,
            typename std::conditional<AMODE == A_CONV_C32, ConvC32, ConvGen>::type>::type>::type AGen;
    typedef typename std::conditional<BVEC, LinearVec, LinearScalar>::type BGen;
    AGen ag[T::A_UNITS];
    BGen bg[T::B_UNITS];
    int a_dst[T::A_UNITS], b_dst[T::B_UNITS];  // LDS byte offset of digit 0 inside a stage
#pragma unroll
    for (int i = 0; i < T::A_UNITS; ++i) {
        const int u = tid + i * T::NT, q = u & 3, row = (u >> 2) % T::BM, jh = (u >> 2) / T::BM;
        if constexpr (AMODE == A_LINEAR_VEC || AMODE == A_LINEAR_SCALAR) ag[i].init(p, row, rows_m, (u32)p.lda, q, jh);
        else ag[i].init(p, m0, row, rows_m, q, jh);
        a_dst[i] = jh * T::A_RS + row * 16 + q * 4;
    }
#pragma unroll
    for (int i = 0; i < T::B_UNITS; ++i) {
        const int u = tid + i * T::NT, q = u & 3, row = (u >> 2) % T::BN, jh = (u >> 2) / T::BN;
        bg[i].init(p, row, rows_n, (u32)p.K, q, jh);
        b_dst[i] = T::A_BYTES + jh * T::B_RS + row * 16 + q * 4;
    }

    u4 ra[T::A_UNITS][2], rwa[T::B_UNITS][2], rwb[T::B_UNITS][2];

    auto load_a = [&](__amdgpu_buffer_rsrc_t rs, int ks) {
        if constexpr (AMODE == A_CONV_C32) {
            ag[0].begin_kstep(p, ks);
#pragma unroll
            for (int i = 0; i < T::A_UNITS; ++i) {
                ag[i].r = ag[0].r; ag[i].s = ag[0].s; ag[i].tap_off = ag[0].tap_off;
                ag[i].load(p, rs, ra[i]);
            }
        } else if constexpr (AMODE == A_CONV_GEN) {
#pragma unroll
            for (int i = 0; i < T::A_UNITS; ++i) ag[i].load(p, rs, ks, ra[i]);
        } else {
#pragma unroll
            for (int i = 0; i < T::A_UNITS; ++i) ag[i].load(rs, ks, (u32)p.K, ra[i]);
        }
    };
    auto load_b = [&](__amdgpu_buffer_rsrc_t rs, int ks, u4 (*dst)[2]) {
#pragma unroll
        for (int i = 0; i < T::B_UNITS; ++i) bg[i].load(rs, ks, (u32)p.K, dst[i]);
    };
    auto store_a = [&](char* stage) {
#pragma unroll
        for (int i = 0; i < T::A_UNITS; ++i) split_store<T::A_RS>(ra[i][0], ra[i][1], stage + a_dst[i]);
    };
    auto store_b = [&](char* stage, bool sum) {
#pragma unroll
        for (int i = 0; i < T::B_UNITS; ++i) {
            u4 v0 = rwa[i][0], v1 = rwa[i][1];
            if (sum) { v0 = add64x2(v0, rwb[i][0]); v1 = add64x2(v1, rwb[i][1]); }
            split_store<T::B_RS>(v0, v1, stage + b_dst[i]);
        }
    };

    const int a_frag = h * T::A_RS + (wm * SM * 32 + r32) * 16;
    const int b_frag = T::A_BYTES + h * T::B_RS + (wn * SN * 32 + r32) * 16;

    v16i acc[SM][SN][8];

    auto compute = [&](const char* stage) {
        v4i bf[SN][8];
#pragma unroll
        for (int sn = 0; sn < SN; ++sn)
#pragma unroll
            for (int m = 0; m < 8; ++m)
                bf[sn][m] = *reinterpret_cast<const v4i*>(stage + b_frag + m * 2 * T::B_RS + sn * 512);
#pragma unroll
        for (int l = 0; l < 8; ++l) {
            v4i af[SM];
#pragma unroll
            for (int sm = 0; sm < SM; ++sm)
                af[sm] = *reinterpret_cast<const v4i*>(stage + a_frag + l * 2 * T::A_RS + sm * 512);
#pragma unroll
            for (int m = 0; m + l < 8; ++m)
#pragma unroll
                for (int sm = 0; sm < SM; ++sm)
#pragma unroll
                    for (int sn = 0; sn < SN; ++sn)
                        acc[sm][sn][l + m] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
                            af[sm], bf[sn][m], acc[sm][sn][l + m], 0, 0, 0);
        }
    };

    char* const st0 = lds;
    char* const st1 = lds + T::STAGE;
    const int nk = (int)((p.K + 31) / 32);

    for (int kb = 0, seg = 0; kb < nk; kb += SEG_KSTEPS, ++seg) {
        const int ke = kb + SEG_KSTEPS < nk ? kb + SEG_KSTEPS : nk;
#pragma unroll
        for (int sm = 0; sm < SM; ++sm)
#pragma unroll
            for (int sn = 0; sn < SN; ++sn)
#pragma unroll
                for (int s = 0; s < 8; ++s)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[sm][sn][s][i] = 0;

        // even half-step of the first slice
        load_a(rs_xa, kb);
        load_b(rs_wa, kb, rwa);
        load_b(rs_wb, kb, rwb);
        store_a(st0);
        store_b(st0, true);
        __syncthreads();

        for (int ks = kb; ks < ke; ++ks) {
            // even: x_a against w_a + w_b, while the odd half-step's words arrive
            load_a(rs_xb, ks);
            load_b(rs_wa, ks, rwa);
            compute(st0);
            store_a(st1);
            store_b(st1, false);
            __syncthreads();
            // odd: x_b against w_a, while the next slice's words arrive
            const bool more = ks + 1 < ke;
            if (more) {
                load_a(rs_xa, ks + 1);
                load_b(rs_wa, ks + 1, rwa);
                load_b(rs_wb, ks + 1, rwb);
            }
            compute(st1);
            if (more) {
                store_a(st0);
                store_b(st0, true);
            }
            __syncthreads();
        }

        // fold: z (+)= sum_s sext(P_s) << 8s.  P_4..P_7 only reach bits 32..63.
#pragma unroll
        for (int sm = 0; sm < SM; ++sm)
#pragma unroll
            for (int sn = 0; sn < SN; ++sn) {
                const int col = n0 + (wn * SN + sn) * 32 + r32;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int row = m0 + (wm * SM + sm) * 32 + 8 * (i / 4) + 4 * h + (i % 4);
                    u64 v = (u64)(int64_t)acc[sm][sn][0][i];
                    v += (u64)(int64_t)acc[sm][sn][1][i] << 8;
                    v += (u64)(int64_t)acc[sm][sn][2][i] << 16;
                    v += (u64)(int64_t)acc[sm][sn][3][i] << 24;
                    const u32 hi = (u32)acc[sm][sn][4][i] + ((u32)acc[sm][sn][5][i] << 8) +
                                   ((u32)acc[sm][sn][6][i] << 16) + ((u32)acc[sm][sn][7][i] << 24);
                    v += (u64)hi << 32;
                    if (row < p.M && col < p.N) {
                        u64* dst = p.z + (u64)row * (u64)p.N + (u64)col;
                        if (seg > 0) v += *dst;
                        *dst = v;
                    }
                }
            }
    }
}

// ---------------------------------------------------------------------------
template <class T, int AMODE, bool BVEC>
static hipError_t launch(const GemmParams& p, hipStream_t stream) {
    const int64_t tiles_m = (p.M + T::BM - 1) / T::BM, tiles_n = (p.N + T::BN - 1) / T::BN;
    GemmParams q = p;
    q.group_m = tiles_n >= 8 ? 4 : (tiles_n >= 2 ? 8 : 32);
    hipLaunchKernelGGL((share_gemm_kernel<T, AMODE, BVEC>), dim3((unsigned)(tiles_m * tiles_n)), dim3(T::NT), 0,
                       stream, q);
    return hipGetLastError();
}

hipError_t launch_share_gemm(const GemmParams& p, int amode, bool bvec, hipStream_t stream) {
    typedef Tile<4, 2, 1, 1> T;  // 8 waves, 128 x 64 block tile, 32 x 32 per wave
    switch (amode) {
        case A_LINEAR_VEC:    return launch<T, A_LINEAR_VEC, true>(p, stream);
        case A_LINEAR_SCALAR: return launch<T, A_LINEAR_SCALAR, false>(p, stream);
        case A_CONV_C32:      return launch<T, A_CONV_C32, true>(p, stream);
        case A_CONV_GEN:
            return bvec ? launch<T, A_CONV_GEN, true>(p, stream) : launch<T, A_CONV_GEN, false>(p, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace cg
