// C-ABI entry points declared in include/cg.h: host-side validation, choice of
// the address generator, and the element-wise share operations.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <mutex>

#include "cg.h"
#include "prf.h"
#include "share_gemm.h"

namespace {

typedef uint64_t u64;

const int64_t MAX_DIM = 0x7FFFFFFF;      // M, N as 32-bit ints in the kernel
const int64_t MAX_ROW_WORDS = 1 << 20;   // K: MAX_TILE_ROWS rows of K words stay below 2^31 bytes
const int64_t MAX_LONG_ROW_WORDS = (int64_t)1 << 30;   // K of the matrix products: slice indices stay 32-bit
const int64_t MAX_VIEW_BYTES = 0x7FFFFFFF;

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// do [a, a+na) and [b, b+nb) (bytes) intersect?
bool overlap(const void* a, u64 na, const void* b, u64 nb) {
    const uintptr_t pa = reinterpret_cast<uintptr_t>(a), pb = reinterpret_cast<uintptr_t>(b);
    return pa < pb + nb && pb < pa + na;
}

// element-wise calls: identical pointers are fine (in place), partial overlap is not
bool bad_overlap(const void* out, const void* in, u64 bytes) {
    return out != in && overlap(out, bytes, in, bytes);
}

bool mul_overflows(int64_t a, int64_t b, int64_t* out) { return __builtin_mul_overflow(a, b, out); }

// ---- element-wise kernels: pure streaming, 16 bytes per lane per access ------
typedef unsigned long long ull2 __attribute__((ext_vector_type(2)));

const int EW_THREADS = 256;

// Each thread handles EW_UNROLL 16-byte pairs per trip, one block-width apart, so
// that several independent loads per stream are in flight before the first add.
const int EW_UNROLL = 4;

template <class F>
__global__ __launch_bounds__(EW_THREADS) void ew_kernel(size_t n, F f) {
    const size_t n2 = n >> 1;
    const size_t chunk = (size_t)EW_THREADS * EW_UNROLL;
    const size_t stride = (size_t)gridDim.x * chunk;
    for (size_t base = (size_t)blockIdx.x * chunk; base < n2; base += stride) {
        const size_t i0 = base + threadIdx.x;
        if (base + chunk <= n2) {
            f.template pairs<EW_UNROLL>(i0, EW_THREADS);
        } else {
#pragma unroll
            for (int u = 0; u < EW_UNROLL; ++u)
                if (i0 + (size_t)u * EW_THREADS < n2) f.template pairs<1>(i0 + (size_t)u * EW_THREADS, EW_THREADS);
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0 && (n & 1)) f.one(n - 1);
}

template <class F>
__global__ __launch_bounds__(EW_THREADS) void ew_kernel_scalar(size_t n, F f) {
    const size_t stride = (size_t)gridDim.x * EW_THREADS;
    for (size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < n; i += stride) f.one(i);
}

// streaming (non-temporal) 16-byte accesses: every element is touched once
__device__ __forceinline__ ull2 ld2(const u64* p, size_t i) {
    return __builtin_nontemporal_load(reinterpret_cast<const ull2*>(p) + i);
}
__device__ __forceinline__ void st2(u64* p, size_t i, ull2 v) {
    __builtin_nontemporal_store(v, reinterpret_cast<ull2*>(p) + i);
}

struct AddOp {  // (za, zb) = (xa + ya, xb + yb)
    const u64 *xa, *xb, *ya, *yb;
    u64 *za, *zb;
    template <int U>
    __device__ void pairs(size_t i, size_t step) const {
        ull2 a[U], b[U], c[U], d[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            a[u] = ld2(xa, i + u * step); c[u] = ld2(ya, i + u * step);
            b[u] = ld2(xb, i + u * step); d[u] = ld2(yb, i + u * step);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            st2(za, i + u * step, a[u] + c[u]);
            st2(zb, i + u * step, b[u] + d[u]);
        }
    }
    __device__ void one(size_t i) const {
        const u64 a = xa[i] + ya[i], b = xb[i] + yb[i];
        za[i] = a;
        zb[i] = b;
    }
};

struct MulPublicOp {  // (za, zb) = (alpha xa, alpha xb)
    const u64 *xa, *xb;
    u64 alpha;
    u64 *za, *zb;
    template <int U>
    __device__ void pairs(size_t i, size_t step) const {
        ull2 a[U], b[U];
#pragma unroll
        for (int u = 0; u < U; ++u) { a[u] = ld2(xa, i + u * step); b[u] = ld2(xb, i + u * step); }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            st2(za, i + u * step, a[u] * alpha);
            st2(zb, i + u * step, b[u] * alpha);
        }
    }
    __device__ void one(size_t i) const {
        const u64 a = xa[i] * alpha, b = xb[i] * alpha;
        za[i] = a;
        zb[i] = b;
    }
};

struct AddPublicOp {  // (za, zb) = (xa + ga, xb + gb)
    const u64 *xa, *xb;
    u64 ga, gb;
    u64 *za, *zb;
    template <int U>
    __device__ void pairs(size_t i, size_t step) const {
        ull2 a[U], b[U];
#pragma unroll
        for (int u = 0; u < U; ++u) { a[u] = ld2(xa, i + u * step); b[u] = ld2(xb, i + u * step); }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            st2(za, i + u * step, a[u] + ga);
            st2(zb, i + u * step, b[u] + gb);
        }
    }
    __device__ void one(size_t i) const {
        const u64 a = xa[i] + ga, b = xb[i] + gb;
        za[i] = a;
        zb[i] = b;
    }
};

struct ReconstructOp {  // out = s0 + s1 + s2
    const u64 *s0, *s1, *s2;
    u64* out;
    template <int U>
    __device__ void pairs(size_t i, size_t step) const {
        ull2 a[U], b[U], c[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            a[u] = ld2(s0, i + u * step); b[u] = ld2(s1, i + u * step); c[u] = ld2(s2, i + u * step);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) st2(out, i + u * step, a[u] + b[u] + c[u]);
    }
    __device__ void one(size_t i) const { out[i] = s0[i] + s1[i] + s2[i]; }
};

// z[j] = x_a[j] y_a[j'] + x_b[j] y_a[j'] + x_a[j] y_b[j'],  j' = j mod period
// (two ring products per element by distributivity: x_a (y_a + y_b) + x_b y_a)
struct PartyMulOp {
    const u64 *xa, *xb, *ya, *yb;
    u64* z;
    size_t period;   // in elements; the pair path requires it to be even (or equal to n)
    template <int U>
    __device__ void pairs(size_t i, size_t step) const {
        const size_t hp = period >> 1;
        ull2 a[U], b[U], c[U], d[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t k = i + u * step, kp = k % hp;
            a[u] = ld2(xa, k); b[u] = ld2(xb, k);
            c[u] = reinterpret_cast<const ull2*>(ya)[kp];
            d[u] = reinterpret_cast<const ull2*>(yb)[kp];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) st2(z, i + u * step, a[u] * (c[u] + d[u]) + b[u] * c[u]);
    }
    __device__ void one(size_t i) const {
        const size_t ip = i % period;
        z[i] = xa[i] * (ya[ip] + yb[ip]) + xb[i] * ya[ip];
    }
};

// (za, zb) = (xa + ba[j'], xb + bb[j']), j' = j mod period: a bias share broadcast over the rows
struct BiasAddOp {
    const u64 *xa, *xb, *ba, *bb;
    u64 *za, *zb;
    size_t period;   // in elements; the pair path requires it to be even
    template <int U>
    __device__ void pairs(size_t i, size_t step) const {
        const size_t hp = period >> 1;
        ull2 a[U], b[U], c[U], d[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t k = i + u * step, kp = k % hp;
            a[u] = ld2(xa, k); b[u] = ld2(xb, k);
            c[u] = reinterpret_cast<const ull2*>(ba)[kp];
            d[u] = reinterpret_cast<const ull2*>(bb)[kp];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            st2(za, i + u * step, a[u] + c[u]);
            st2(zb, i + u * step, b[u] + d[u]);
        }
    }
    __device__ void one(size_t i) const {
        const size_t ip = i % period;
        const u64 a = xa[i] + ba[ip], b = xb[i] + bb[ip];
        za[i] = a;
        zb[i] = b;
    }
};

// Column sums of both components of x [rows, cols] into zero-filled za, zb [cols].  A block covers 64
// columns (one per lane, so a wave reads 512 contiguous bytes of a row) and a slice of the rows; its
// four waves take rows in turn, their partial sums meet in LDS and one wave adds them to the output
// atomically (integer sums mod 2^64 do not depend on the order).
__global__ __launch_bounds__(256) void col_sum_kernel(const u64* __restrict__ xa, const u64* __restrict__ xb,
                                                      u64* __restrict__ za, u64* __restrict__ zb, size_t rows,
                                                      size_t cols) {
    __shared__ u64 part[2][4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t c = (size_t)blockIdx.x * 64 + lane;
    u64 sa = 0, sb = 0;
    if (c < cols) {
        const size_t stride = (size_t)gridDim.y * 4;
        size_t r = (size_t)blockIdx.y * 4 + wave;
        for (; r + 3 * stride < rows; r += 4 * stride) {   // four independent loads per stream in flight
            const u64 a0 = xa[r * cols + c], a1 = xa[(r + stride) * cols + c], a2 = xa[(r + 2 * stride) * cols + c],
                      a3 = xa[(r + 3 * stride) * cols + c];
            const u64 b0 = xb[r * cols + c], b1 = xb[(r + stride) * cols + c], b2 = xb[(r + 2 * stride) * cols + c],
                      b3 = xb[(r + 3 * stride) * cols + c];
            sa += (a0 + a1) + (a2 + a3);
            sb += (b0 + b1) + (b2 + b3);
        }
        for (; r < rows; r += stride) {
            sa += xa[r * cols + c];
            sb += xb[r * cols + c];
        }
    }
    part[0][wave][lane] = sa;
    part[1][wave][lane] = sb;
    __syncthreads();
    if (wave == 0 && c < cols) {
        sa = part[0][0][lane] + part[0][1][lane] + part[0][2][lane] + part[0][3][lane];
        sb = part[1][0][lane] + part[1][1][lane] + part[1][2][lane] + part[1][3][lane];
        atomicAdd(reinterpret_cast<unsigned long long*>(za + c), (unsigned long long)sa);
        atomicAdd(reinterpret_cast<unsigned long long*>(zb + c), (unsigned long long)sb);
    }
}

__global__ __launch_bounds__(256) void zero2_kernel(u64* a, u64* b, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        a[i] = 0;
        b[i] = 0;
    }
}

// ---- binary (XOR) replicated shares: 64 independent bits per word ----------------
struct BXorOp {  // (za, zb) = (xa ^ ya, xb ^ yb)
    const u64 *xa, *xb, *ya, *yb;
    u64 *za, *zb;
    template <int U>
    __device__ void pairs(size_t i, size_t step) const {
        ull2 a[U], b[U], c[U], d[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            a[u] = ld2(xa, i + u * step); c[u] = ld2(ya, i + u * step);
            b[u] = ld2(xb, i + u * step); d[u] = ld2(yb, i + u * step);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            st2(za, i + u * step, a[u] ^ c[u]);
            st2(zb, i + u * step, b[u] ^ d[u]);
        }
    }
    __device__ void one(size_t i) const {
        const u64 a = xa[i] ^ ya[i], b = xb[i] ^ yb[i];
        za[i] = a;
        zb[i] = b;
    }
};

// z = (x_a & y_a) ^ (x_b & y_a) ^ (x_a & y_b) = (x_a & (y_a ^ y_b)) ^ (x_b & y_a)
struct BAndOp {
    const u64 *xa, *xb, *ya, *yb;
    u64* z;
    template <int U>
    __device__ void pairs(size_t i, size_t step) const {
        ull2 a[U], b[U], c[U], d[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            a[u] = ld2(xa, i + u * step); c[u] = ld2(ya, i + u * step);
            b[u] = ld2(xb, i + u * step); d[u] = ld2(yb, i + u * step);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) st2(z, i + u * step, (a[u] & (c[u] ^ d[u])) ^ (b[u] & c[u]));
    }
    __device__ void one(size_t i) const { z[i] = (xa[i] & (ya[i] ^ yb[i])) ^ (xb[i] & ya[i]); }
};

// One stage of the parallel-prefix adder on (propagate, generate) words:
//   g' = g_a ^ and3(p, g << s),  p' = and3(p, p << s),  and3 = the three-term AND above.
struct PrefixStageOp {
    const u64 *pa, *pb, *ga, *gb;
    u64 *p_out, *g_out;  // p_out may be null (last stage)
    int s;
    template <int U>
    __device__ void pairs(size_t i, size_t step) const {
        ull2 a[U], b[U], c[U], d[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            a[u] = ld2(pa, i + u * step); c[u] = ld2(ga, i + u * step);
            b[u] = ld2(pb, i + u * step); d[u] = ld2(gb, i + u * step);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const ull2 gsa = c[u] << s, gsb = d[u] << s;
            st2(g_out, i + u * step, c[u] ^ (a[u] & (gsa ^ gsb)) ^ (b[u] & gsa));
            if (p_out) {
                const ull2 psa = a[u] << s, psb = b[u] << s;
                st2(p_out, i + u * step, (a[u] & (psa ^ psb)) ^ (b[u] & psa));
            }
        }
    }
    __device__ void one(size_t i) const {
        const u64 a = pa[i], b = pb[i], c = ga[i], d = gb[i];
        const u64 gsa = c << s, gsb = d << s;
        g_out[i] = c ^ (a & (gsa ^ gsb)) ^ (b & gsa);
        if (p_out) {
            const u64 psa = a << s, psb = b << s;
            p_out[i] = (a & (psa ^ psb)) ^ (b & psa);
        }
    }
};

// Carry-save (full) adder on three binary sharings, one party's local step: sum pair S = A ^ B ^ C and the
// party's XOR share of the carry ((A ^ C) & (B ^ C)) ^ C (three-term AND, own component of C added).
struct CsaOp {
    const u64 *aa, *ab, *ba, *bb, *ca, *cb;  // a null input is a component that is zero everywhere
    u64 *sa, *sb, *carry;
    static __device__ __forceinline__ ull2 in2(const u64* p, size_t k) { return p ? ld2(p, k) : ull2{0, 0}; }
    template <int U>
    __device__ void pairs(size_t i, size_t step) const {
        ull2 a0[U], a1[U], b0[U], b1[U], c0[U], c1[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t k = i + u * step;
            a0[u] = in2(aa, k); a1[u] = in2(ab, k); b0[u] = in2(ba, k);
            b1[u] = in2(bb, k); c0[u] = in2(ca, k); c1[u] = in2(cb, k);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t k = i + u * step;
            const ull2 x0 = a0[u] ^ c0[u], x1 = a1[u] ^ c1[u], y0 = b0[u] ^ c0[u], y1 = b1[u] ^ c1[u];
            st2(sa, k, x0 ^ b0[u]);
            st2(sb, k, x1 ^ b1[u]);
            st2(carry, k, (x0 & (y0 ^ y1)) ^ (x1 & y0) ^ c0[u]);
        }
    }
    __device__ void one(size_t k) const {
        const u64 c0 = ca ? ca[k] : 0, c1 = cb ? cb[k] : 0, b0 = ba ? ba[k] : 0, b1 = bb ? bb[k] : 0;
        const u64 x0 = (aa ? aa[k] : 0) ^ c0, x1 = (ab ? ab[k] : 0) ^ c1, y0 = b0 ^ c0, y1 = b1 ^ c1;
        sa[k] = x0 ^ b0;
        sb[k] = x1 ^ b1;
        carry[k] = (x0 & (y0 ^ y1)) ^ (x1 & y0) ^ c0;
    }
};

// Half adder on two binary sharings: propagate pair P = S ^ T and the party's XOR share of generate S & T.
struct HalfAdderOp {
    const u64 *sa, *sb, *ta, *tb;
    u64 *pa, *pb, *g;
    template <int U>
    __device__ void pairs(size_t i, size_t step) const {
        ull2 s0[U], s1[U], t0[U], t1[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t k = i + u * step;
            s0[u] = ld2(sa, k); s1[u] = ld2(sb, k); t0[u] = ld2(ta, k); t1[u] = ld2(tb, k);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t k = i + u * step;
            st2(pa, k, s0[u] ^ t0[u]);
            st2(pb, k, s1[u] ^ t1[u]);
            st2(g, k, (s0[u] & (t0[u] ^ t1[u])) ^ (s1[u] & t0[u]));
        }
    }
    __device__ void one(size_t k) const {
        const u64 s0 = sa[k], s1 = sb[k], t0 = ta[k], t1 = tb[k];
        pa[k] = s0 ^ t0;
        pb[k] = s1 ^ t1;
        g[k] = (s0 & (t0 ^ t1)) ^ (s1 & t0);
    }
};

// One level of the carry tree on bit planes: inputs [2k, m] words, outputs [k, m]; output plane j merges the
// neighbouring segments hi = plane 2j+1 and lo = plane 2j:
//   g' = g_hi ^ and3(p_hi, g_lo),  p' = and3(p_hi, p_lo),  and3 = the three-term AND on the pairs.
struct CarryLevelOp {
    const u64 *pa, *pb, *ga, *gb;
    u64 *p_out, *g_out;  // p_out may be null (root level)
    size_t m;            // words per plane; the pair path requires it to be even
    template <int U>
    __device__ void pairs(size_t i, size_t step) const {
        const size_t hm = m >> 1;
        ull2 ph_a[U], ph_b[U], gh_a[U], pl_a[U], pl_b[U], gl_a[U], gl_b[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t o = i + u * step, j = o / hm, w = o - j * hm;
            const size_t hi = (2 * j + 1) * hm + w, lo = 2 * j * hm + w;
            ph_a[u] = ld2(pa, hi); ph_b[u] = ld2(pb, hi); gh_a[u] = ld2(ga, hi);
            gl_a[u] = ld2(ga, lo); gl_b[u] = ld2(gb, lo);
            if (p_out) { pl_a[u] = ld2(pa, lo); pl_b[u] = ld2(pb, lo); }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            st2(g_out, i + u * step, gh_a[u] ^ (ph_a[u] & (gl_a[u] ^ gl_b[u])) ^ (ph_b[u] & gl_a[u]));
            if (p_out) st2(p_out, i + u * step, (ph_a[u] & (pl_a[u] ^ pl_b[u])) ^ (ph_b[u] & pl_a[u]));
        }
    }
    __device__ void one(size_t o) const {
        const size_t j = o / m, w = o - j * m;
        const size_t hi = (2 * j + 1) * m + w, lo = 2 * j * m + w;
        const u64 a = pa[hi], b = pb[hi];
        g_out[o] = ga[hi] ^ (a & (ga[lo] ^ gb[lo])) ^ (b & ga[lo]);
        if (p_out) p_out[o] = (a & (pa[lo] ^ pb[lo])) ^ (b & pa[lo]);
    }
};

// 64 x 64 bit transpose: plane b, word w, bit e = bit b of src[64 w + e].  A wave takes BT_BLOCKS blocks of 64
// words per trip.  Lane e loads its word of a block (512 contiguous bytes per block); the block is transposed in
// registers by the recursive scheme (swap the off-diagonal j x j sub-blocks for j = 32, 16, .., 1, each step one
// exchange with lane e ^ j and a masked merge), after which lane b holds the word of plane b.  The words then
// cross the wave's own LDS tile [plane][block], so that each half of the wave stores 256 contiguous bytes of
// one plane instead of every lane 8 bytes of its own.
template <int J>
__device__ __forceinline__ u64 transpose_step(u64 x, int lane) {
    // bits whose index has bit J clear
    constexpr u64 mask = J == 32 ? 0x00000000FFFFFFFFull : J == 16 ? 0x0000FFFF0000FFFFull
                       : J == 8 ? 0x00FF00FF00FF00FFull : J == 4 ? 0x0F0F0F0F0F0F0F0Full
                       : J == 2 ? 0x3333333333333333ull : 0x5555555555555555ull;
    const u64 y = (u64)__shfl_xor((unsigned long long)x, J, 64);
    return (lane & J) ? (((y >> J) & mask) | (x & ~mask)) : ((x & mask) | ((y & mask) << J));
}

__device__ __forceinline__ u64 transpose64_lanes(u64 x, int lane) {
    x = transpose_step<32>(x, lane);
    x = transpose_step<16>(x, lane);
    x = transpose_step<8>(x, lane);
    x = transpose_step<4>(x, lane);
    x = transpose_step<2>(x, lane);
    return transpose_step<1>(x, lane);
}

constexpr int BT_BLOCKS = 32;            // 64-word blocks per wave and trip
constexpr int BT_PITCH = BT_BLOCKS + 1;  // words between planes in the LDS tile: consecutive lanes hit distinct banks

__global__ __launch_bounds__(256) void bit_transpose_kernel(const u64* __restrict__ src, u64* __restrict__ dst, size_t m) {
    __shared__ u64 tile_all[4][64 * BT_PITCH];
    const int lane = threadIdx.x & 63;
    u64* tile = tile_all[threadIdx.x >> 6];  // private to the wave: no block barrier anywhere
    const size_t wave = ((size_t)blockIdx.x * 256 + threadIdx.x) >> 6, waves = ((size_t)gridDim.x * 256) >> 6;
    const int half = lane >> 5, col = lane & 31;
    for (size_t w0 = wave * BT_BLOCKS; w0 < m; w0 += waves * BT_BLOCKS) {
        u64 mine[BT_BLOCKS];
#pragma unroll
        for (int k = 0; k < BT_BLOCKS; ++k) {
            const size_t w = w0 + k;
            mine[k] = w < m ? src[64 * w + lane] : 0;       // uniform per k: whole blocks only
        }
#pragma unroll
        for (int k = 0; k < BT_BLOCKS; ++k) tile[lane * BT_PITCH + k] = transpose64_lanes(mine[k], lane);
        // the tile is read by other lanes of the same wave: LDS operations of a wave complete in order
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const bool in = w0 + col < m;
#pragma unroll 8
        for (int pl = 0; pl < 64; pl += 2) {
            const u64 v = tile[(pl + half) * BT_PITCH + col];
            if (in) dst[(size_t)(pl + half) * m + w0 + col] = v;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();    // the next trip overwrites the tile
    }
}

// out[i] = bit (i % 64) of plane[i / 64]
__global__ __launch_bounds__(256) void bits_unpack_kernel(const u64* __restrict__ plane, u64* __restrict__ out, size_t n) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) out[i] = (plane[i >> 6] >> (i & 63)) & 1;
}

// One thread per output pixel and channel pair: sums the window of both components.
__global__ __launch_bounds__(256) void sum_pool_kernel(const u64* __restrict__ xa, const u64* __restrict__ xb,
                                                       u64* __restrict__ za, u64* __restrict__ zb,
                                                       int B, int H, int W, int C, int Ho, int Wo, int kh, int kw,
                                                       int sh, int sw, int ph, int pw, int vec) {
    const int cw = vec ? C / 2 : C;   // channel groups per pixel
    const size_t total = (size_t)B * Ho * Wo * cw;
    for (size_t t = (size_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (size_t)gridDim.x * 256) {
        const int cg_ = (int)(t % cw);
        size_t pix = t / cw;
        const int wo = (int)(pix % Wo);
        pix /= Wo;
        const int ho = (int)(pix % Ho), b = (int)(pix / Ho);
        ull2 sa = {0, 0}, sb = {0, 0};
        for (int r = 0; r < kh; ++r) {
            const int hi = ho * sh - ph + r;
            if (hi < 0 || hi >= H) continue;
            for (int s = 0; s < kw; ++s) {
                const int wi = wo * sw - pw + s;
                if (wi < 0 || wi >= W) continue;
                const size_t off = (((size_t)b * H + hi) * W + wi) * C;
                if (vec) {
                    sa += reinterpret_cast<const ull2*>(xa + off)[cg_];
                    sb += reinterpret_cast<const ull2*>(xb + off)[cg_];
                } else {
                    sa.x += xa[off + cg_];
                    sb.x += xb[off + cg_];
                }
            }
        }
        const size_t o = (((size_t)b * Ho + ho) * Wo + wo) * C;
        if (vec) {
            reinterpret_cast<ull2*>(za + o)[cg_] = sa;
            reinterpret_cast<ull2*>(zb + o)[cg_] = sb;
        } else {
            za[o + cg_] = sa.x;
            zb[o + cg_] = sb.x;
        }
    }
}

template <class F>
cg_status launch_ew(size_t n, bool vec, const F& f, void* stream) {
    if (n == 0) return CG_OK;
    const size_t work = vec ? ((n + 1) / 2 + EW_UNROLL - 1) / EW_UNROLL : n;
    size_t blocks = (work + EW_THREADS - 1) / EW_THREADS;
    const size_t cap = 256 * 16;  // 16 resident blocks per compute unit, grid-stride beyond that
    if (blocks > cap) blocks = cap;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (vec) hipLaunchKernelGGL(ew_kernel<F>, dim3((unsigned)blocks), dim3(EW_THREADS), 0, s, n, f);
    else hipLaunchKernelGGL(ew_kernel_scalar<F>, dim3((unsigned)blocks), dim3(EW_THREADS), 0, s, n, f);
    return hipGetLastError() == hipSuccess ? CG_OK : CG_ERR_DEVICE;
}

cg_status check_ptrs(const void* const* ptrs, int count) {
    for (int i = 0; i < count; ++i)
        if (!ptrs[i]) return CG_ERR_NULL;
    for (int i = 0; i < count; ++i)
        if (!aligned(ptrs[i], 8)) return CG_ERR_ALIGN;
    return CG_OK;
}

bool all_aligned16(const void* const* ptrs, int count) {
    for (int i = 0; i < count; ++i)
        if (!aligned(ptrs[i], 16)) return false;
    return true;
}

cg_status check_product_ptrs(const u64* x_i, const u64* x_ip1, const u64* y_i, const u64* y_ip1, u64* z_i,
                             u64 x_bytes, u64 y_bytes, u64 z_bytes) {
    const void* ptrs[5] = {x_i, x_ip1, y_i, y_ip1, z_i};
    if (cg_status st = check_ptrs(ptrs, 5)) return st;
    if (overlap(z_i, z_bytes, x_i, x_bytes) || overlap(z_i, z_bytes, x_ip1, x_bytes) ||
        overlap(z_i, z_bytes, y_i, y_bytes) || overlap(z_i, z_bytes, y_ip1, y_bytes))
        return CG_ERR_ALIAS;
    return CG_OK;
}

}  // namespace

extern "C" {

const char* cg_status_string(cg_status s) {
    switch (s) {
        case CG_OK: return "CG_OK";
        case CG_ERR_NULL: return "CG_ERR_NULL: a required pointer is NULL";
        case CG_ERR_SHAPE: return "CG_ERR_SHAPE: bad or overflowing dimensions";
        case CG_ERR_ALIGN: return "CG_ERR_ALIGN: pointer not 8-byte aligned";
        case CG_ERR_ALIAS: return "CG_ERR_ALIAS: output overlaps an input";
        case CG_ERR_UNSUPPORTED: return "CG_ERR_UNSUPPORTED: shape outside the kernels' addressing range";
        case CG_ERR_DEVICE: return "CG_ERR_DEVICE: HIP launch error";
        case CG_ERR_WORKSPACE: return "CG_ERR_WORKSPACE: scratch memory smaller than the product needs (cg_*_workspace_bytes())";
    }
    return "unknown cg_status";
}

int cg_version(void) { return 100; }

}  // extern "C"

namespace {

// What a validated call resolves to.
struct Plan {
    cg::GemmParams p;
    int amode;        // address generator of the direct route
    int bmode;
    bool planes_ok;   // the digit-plane route applies
    bool planes_conv; // ... with the patch gather
    int64_t x_rows, x_k;  // left operand seen as [x_rows, x_k] words for the plane conversion
    u64 xp_bytes, wp_bytes;  // bytes of one left / right plane tensor
    u64 x_bytes, w_bytes, z_bytes;
};

u64 round_up(u64 v, u64 a) { return (v + a - 1) / a * a; }

// Does the digit route (one conversion launch, then a product kernel without split work) beat the plain
// product for this plan?  Measured on MI355X: the plain kernel runs at about half the published int8 rate (144
// int8 ops per (m, n, k) at 2.45e15 op/s), the product kernel of the digit route saves about 17 % of that time,
// and the conversion moves 32 bytes per operand word at about 6.5 TB/s after a launch of about 5 microseconds.
// The route must win by a margin to be preferred.
bool planes_pay(const Plan& pl) {
    if (!pl.planes_ok) return false;
    const double mnk = (double)pl.p.M * (double)pl.p.N * (double)pl.p.K;
    const double words = (double)pl.x_rows * (double)pl.x_k + (double)pl.p.N * (double)pl.p.K;
    return 0.17 * 144.0 * mnk / 2.45e15 > 1.15 * (32.0 * words / 6.5e12 + 5.0e-6);
}

u64 plan_workspace_bytes(const Plan& pl) {
    return pl.planes_ok ? 2 * round_up(pl.xp_bytes, 256) + 2 * round_up(pl.wp_bytes, 256) : 0;
}

cg_status plan_matmul(const uint64_t* x_i, const uint64_t* x_ip1, const uint64_t* y_i, const uint64_t* y_ip1,
                      uint64_t* z_i, int64_t M, int64_t N, int64_t K, bool check_ptrs_too, Plan* out,
                      bool trans_x = false, bool trans_y = false) {
    if (check_ptrs_too && (!x_i || !x_ip1 || !y_i || !y_ip1 || !z_i)) return CG_ERR_NULL;
    if (M < 1 || N < 1 || K < 1) return CG_ERR_SHAPE;
    int64_t mk, nk, mn, tmp;
    if (mul_overflows(M, K, &mk) || mul_overflows(N, K, &nk) || mul_overflows(M, N, &mn) ||
        mul_overflows(mk, 8, &tmp) || mul_overflows(nk, 8, &tmp) || mul_overflows(mn, 8, &tmp))
        return CG_ERR_SHAPE;
    if (check_ptrs_too)
        if (cg_status st = check_product_ptrs(x_i, x_ip1, y_i, y_ip1, z_i, (u64)mk * 8, (u64)nk * 8, (u64)mn * 8))
            return st;
    if (M > MAX_DIM || N > MAX_DIM || K > MAX_LONG_ROW_WORDS) return CG_ERR_UNSUPPORTED;

    Plan pl = {};
    cg::GemmParams& p = pl.p;
    p.x_a = x_i; p.x_b = x_ip1; p.w_a = y_i; p.w_b = y_ip1; p.z = z_i;
    p.M = (int)M; p.N = (int)N; p.K = (int)K; p.lda = (int)K;
    p.x_elems = (u64)mk;
    p.w_elems = (u64)nk;
    p.Ho = p.Wo = 1;
    const void* in[4] = {x_i, x_ip1, y_i, y_ip1};
    const bool vec = (K % 2 == 0) && (!check_ptrs_too || all_aligned16(in, 4));
    pl.amode = trans_x ? cg::A_TRANS : (vec ? cg::A_LINEAR_VEC : cg::A_LINEAR_SCALAR);
    pl.bmode = trans_y ? cg::B_TRANS : (vec ? cg::B_VEC : cg::B_SCALAR);
    if (trans_x && !trans_y && !vec) pl.bmode = cg::B_SCALAR;
    if (!trans_x && trans_y) pl.amode = vec ? cg::A_LINEAR_VEC : cg::A_LINEAR_SCALAR;
    // a transposed operand is addressed slice by slice: 32 rows of its pitch must fit a 2^31-byte view
    if ((trans_x && M > (1 << 22)) || (trans_y && N > (1 << 22))) return CG_ERR_UNSUPPORTED;
    // rows beyond what a buffer view addresses: the row-major operands take the 64-bit generators
    const bool long_rows = K > MAX_ROW_WORDS;
    if (long_rows) {
        if (!trans_x) pl.amode = cg::A_LINEAR_WIDE;
        if (!trans_y) pl.bmode = cg::B_WIDE;
    }
    // (a product of few rows is a few microseconds on the kernel of its own: converting its operands first would
    // cost more than the product)
    pl.planes_ok = vec && !trans_x && !trans_y && !long_rows && !cg::share_gemm_small_applies(p);
    pl.planes_conv = false;
    pl.x_rows = M; pl.x_k = K;
    pl.xp_bytes = cg::planes_bytes(M, K); pl.wp_bytes = cg::planes_bytes(N, K);
    pl.x_bytes = (u64)mk * 8; pl.w_bytes = (u64)nk * 8; pl.z_bytes = (u64)mn * 8;
    *out = pl;
    return CG_OK;
}

// Sizes of a convolution layer, with every product checked against int64 overflow.
struct ConvDims {
    int64_t Ho, Wo, img, x_el, K, w_el, howo, M, z_el;
};

cg_status conv_dims(const cg_conv2d_desc* d, ConvDims* o) {
    if (d->B < 1 || d->H < 1 || d->W < 1 || d->Cin < 1 || d->Cout < 1 || d->kh < 1 || d->kw < 1 ||
        d->stride_h < 1 || d->stride_w < 1 || d->pad_h < 0 || d->pad_w < 0)
        return CG_ERR_SHAPE;
    // keep every intermediate far from int64 overflow
    const int64_t LIM = (int64_t)1 << 40;
    if (d->B > LIM || d->H > LIM || d->W > LIM || d->Cin > LIM || d->Cout > LIM || d->kh > LIM || d->kw > LIM ||
        d->stride_h > LIM || d->stride_w > LIM || d->pad_h > LIM || d->pad_w > LIM)
        return CG_ERR_SHAPE;
    const int64_t span_h = d->H + 2 * d->pad_h - d->kh, span_w = d->W + 2 * d->pad_w - d->kw;
    if (span_h < 0 || span_w < 0) return CG_ERR_SHAPE;
    o->Ho = span_h / d->stride_h + 1;
    o->Wo = span_w / d->stride_w + 1;
    int64_t tmp;
    if (mul_overflows(d->H, d->W, &tmp) || mul_overflows(tmp, d->Cin, &o->img) ||
        mul_overflows(o->img, d->B, &o->x_el) || mul_overflows(d->kh, d->kw, &tmp) ||
        mul_overflows(tmp, d->Cin, &o->K) || mul_overflows(o->K, d->Cout, &o->w_el) ||
        mul_overflows(o->Ho, o->Wo, &o->howo) || mul_overflows(o->howo, d->B, &o->M) ||
        mul_overflows(o->M, d->Cout, &o->z_el) || mul_overflows(o->x_el, 8, &tmp) ||
        mul_overflows(o->w_el, 8, &tmp) || mul_overflows(o->z_el, 8, &tmp))
        return CG_ERR_SHAPE;
    return CG_OK;
}

cg_status plan_conv2d(const uint64_t* x_i, const uint64_t* x_ip1, const uint64_t* w_i, const uint64_t* w_ip1,
                      uint64_t* z_i, const cg_conv2d_desc* d, bool check_ptrs_too, Plan* out) {
    if (!d) return CG_ERR_NULL;
    if (check_ptrs_too && (!x_i || !x_ip1 || !w_i || !w_ip1 || !z_i)) return CG_ERR_NULL;
    ConvDims cd;
    if (cg_status st = conv_dims(d, &cd)) return st;
    const int64_t Ho = cd.Ho, Wo = cd.Wo, img = cd.img, x_el = cd.x_el, K = cd.K, w_el = cd.w_el, howo = cd.howo,
                  M = cd.M, z_el = cd.z_el;
    if (check_ptrs_too)
        if (cg_status st = check_product_ptrs(x_i, x_ip1, w_i, w_ip1, z_i, (u64)x_el * 8, (u64)w_el * 8, (u64)z_el * 8))
            return st;
    if (M > MAX_DIM || d->Cout > MAX_DIM || K > MAX_ROW_WORDS || img > ((int64_t)1 << 27) ||
        d->pad_h > 32767 || d->pad_w > 32767 || d->stride_h > 32767 || d->stride_w > 32767)
        return CG_ERR_UNSUPPORTED;

    Plan pl = {};
    cg::GemmParams& p = pl.p;
    p.x_a = x_i; p.x_b = x_ip1; p.w_a = w_i; p.w_b = w_ip1; p.z = z_i;
    p.M = (int)M; p.N = (int)d->Cout; p.K = (int)K;
    p.x_elems = (u64)x_el;
    p.w_elems = (u64)w_el;
    p.img_elems = (u64)img;
    p.H = (int)d->H; p.W = (int)d->W; p.Cin = (int)d->Cin; p.Ho = (int)Ho; p.Wo = (int)Wo;
    p.kh = (int)d->kh; p.kw = (int)d->kw; p.sh = (int)d->stride_h; p.sw = (int)d->stride_w;
    p.ph = (int)d->pad_h; p.pw = (int)d->pad_w;
    p.div_cin = cg::make_fast_div((uint32_t)d->Cin);
    p.div_kw = cg::make_fast_div((uint32_t)d->kw);

    const void* in[4] = {x_i, x_ip1, w_i, w_ip1};
    const bool a16 = !check_ptrs_too || all_aligned16(in, 4);
    int amode;
    bool bvec = a16 && (K % 2 == 0);
    const bool pointwise = d->kh == 1 && d->kw == 1 && d->stride_h == 1 && d->stride_w == 1 &&
                           d->pad_h == 0 && d->pad_w == 0;
    if (pointwise) {
        // a 1x1, stride-1, unpadded convolution IS the matrix product [B*H*W, Cin] x [Cout, Cin]^T
        p.lda = (int)d->Cin;
        amode = bvec ? cg::A_LINEAR_VEC : cg::A_LINEAR_SCALAR;
        bvec = amode == cg::A_LINEAR_VEC;
    } else {
        // one block's rows touch at most this many consecutive images; their bytes must fit a 2^31 view
        const int64_t span_imgs = (cg::MAX_TILE_ROWS - 1) / howo + 2;
        const int64_t view = (span_imgs < d->B ? span_imgs : d->B) * img * 8;
        if (view > MAX_VIEW_BYTES) return CG_ERR_UNSUPPORTED;
        amode = (a16 && d->Cin % 32 == 0 && d->kh * d->kw <= cg::MAX_MASK_TAPS) ? cg::A_CONV_C32 : cg::A_CONV_GEN;
    }
    pl.amode = amode;
    pl.bmode = bvec ? cg::B_VEC : cg::B_SCALAR;
    if (pointwise) {
        pl.planes_ok = bvec;
        pl.planes_conv = false;
        pl.x_rows = M; pl.x_k = d->Cin;
    } else {
        // (the plane view of a block starts up to 15 pixels ahead of its first image)
        const int64_t span_imgs = (cg::MAX_TILE_ROWS - 1) / howo + 2;
        const int64_t view = (span_imgs < d->B ? span_imgs : d->B) * img * 8 + 16 * d->Cin * 8;
        pl.planes_ok = amode == cg::A_CONV_C32 && view <= MAX_VIEW_BYTES;
        pl.planes_conv = true;
        pl.x_rows = d->B * d->H * d->W; pl.x_k = d->Cin;
    }
    pl.xp_bytes = cg::planes_bytes(pl.x_rows, pl.x_k);
    pl.wp_bytes = cg::planes_bytes(d->Cout, K);
    pl.x_bytes = (u64)x_el * 8; pl.w_bytes = (u64)w_el * 8; pl.z_bytes = (u64)z_el * 8;
    *out = pl;
    return CG_OK;
}

// Input gradient of a convolution layer as a product of the kernel's form: rows are the
// pixels of the layer INPUT, the contraction runs over (tap, output channel), the left
// operand gathers patches of the incoming gradient (zero-interleaved when the layer is
// strided) with padding k - 1 - pad, and the right operand is the filter with its taps
// reversed and its channel roles exchanged, addressed in place.
cg_status plan_conv2d_dgrad(const uint64_t* g_i, const uint64_t* g_ip1, const uint64_t* w_i, const uint64_t* w_ip1,
                            uint64_t* dx_i, const cg_conv2d_desc* d, Plan* out) {
    if (!d || !g_i || !g_ip1 || !w_i || !w_ip1 || !dx_i) return CG_ERR_NULL;
    ConvDims cd;
    if (cg_status st = conv_dims(d, &cd)) return st;
    if (cg_status st = check_product_ptrs(g_i, g_ip1, w_i, w_ip1, dx_i, (u64)cd.z_el * 8, (u64)cd.w_el * 8,
                                          (u64)cd.x_el * 8))
        return st;
    const int64_t taps = d->kh * d->kw;
    const int64_t Kg = taps * d->Cout;                 // contraction length
    const int64_t Mg = d->B * d->H * d->W;             // one row per input pixel
    const int64_t g_img = cd.howo * d->Cout;           // words of one image of the gradient
    if (Mg > MAX_DIM || d->Cin > MAX_DIM || Kg > MAX_ROW_WORDS || g_img > ((int64_t)1 << 27) ||
        d->pad_h > 32767 || d->pad_w > 32767 || d->stride_h > 32767 || d->stride_w > 32767 ||
        d->kh > 32767 || d->kw > 32767)
        return CG_ERR_UNSUPPORTED;

    const bool pointwise = taps == 1 && d->stride_h == 1 && d->stride_w == 1 && d->pad_h == 0 && d->pad_w == 0;
    if (pointwise)  // dX [B*H*W, Cin] = G [B*H*W, Cout] x W, the filter [Cout, Cin] being the right operand stored transposed
        return plan_matmul(g_i, g_ip1, w_i, w_ip1, dx_i, Mg, d->Cin, d->Cout, true, out, false, true);

    Plan pl = {};
    cg::GemmParams& p = pl.p;
    p.x_a = g_i; p.x_b = g_ip1; p.w_a = w_i; p.w_b = w_ip1; p.z = dx_i;
    p.M = (int)Mg; p.N = (int)d->Cin; p.K = (int)Kg;
    p.x_elems = (u64)cd.z_el;
    p.w_elems = (u64)cd.w_el;
    p.img_elems = (u64)g_img;
    // the gathered tensor is the gradient [B, Ho, Wo, Cout]; the "output" grid is the layer input's
    p.H = (int)cd.Ho; p.W = (int)cd.Wo; p.Cin = (int)d->Cout; p.Ho = (int)d->H; p.Wo = (int)d->W;
    p.kh = (int)d->kh; p.kw = (int)d->kw; p.sh = 1; p.sw = 1;
    p.ph = (int)(d->kh - 1 - d->pad_h); p.pw = (int)(d->kw - 1 - d->pad_w);
    p.div_cin = cg::make_fast_div((uint32_t)d->Cout);
    p.div_kw = cg::make_fast_div((uint32_t)d->kw);
    p.dil_h = (int)d->stride_h; p.dil_w = (int)d->stride_w;
    p.div_dil_h = cg::make_fast_div((uint32_t)d->stride_h);
    p.div_dil_w = cg::make_fast_div((uint32_t)d->stride_w);

    // one block's rows touch at most this many consecutive images of the gradient
    const int64_t hw = d->H * d->W;
    const int64_t span_imgs = (cg::MAX_TILE_ROWS - 1) / hw + 2;
    if ((span_imgs < d->B ? span_imgs : d->B) * g_img * 8 > MAX_VIEW_BYTES) return CG_ERR_UNSUPPORTED;

    const void* in[4] = {g_i, g_ip1, w_i, w_ip1};
    const bool strided = d->stride_h != 1 || d->stride_w != 1;
    const bool c32 = !strided && all_aligned16(in, 4) && d->Cout % 32 == 0 && taps * d->Cin <= ((int64_t)1 << 22) &&
                     taps <= cg::MAX_MASK_TAPS;
    if (c32) {
        pl.amode = cg::A_CONV_C32; pl.bmode = cg::B_FLIP_C32;
        // the window covers every tap of the filter and the rows are the pixels in order
        p.flt_kh = p.kh; p.flt_kw = p.kw; p.flt_r0 = 0; p.flt_s0 = 0; p.flt_sh = 1; p.flt_sw = 1;
        p.out_H = (int)d->H; p.out_W = (int)d->W; p.out_h0 = 0; p.out_w0 = 0; p.out_sh = 1; p.out_sw = 1;
        p.div_howo = cg::make_fast_div((uint32_t)hw);
        p.div_wo = cg::make_fast_div((uint32_t)d->W);
    } else {
        // every word of the filter is addressed from one view
        if (cd.w_el * 8 > MAX_VIEW_BYTES) return CG_ERR_UNSUPPORTED;
        pl.amode = strided ? cg::A_CONV_DIL : cg::A_CONV_GEN;
        pl.bmode = cg::B_FLIP_GEN;
    }
    pl.x_bytes = (u64)cd.z_el * 8; pl.w_bytes = (u64)cd.w_el * 8; pl.z_bytes = (u64)cd.x_el * 8;
    *out = pl;
    return CG_OK;
}

// Input gradient of a strided convolution, one phase.  Input pixel h = a + stride*i meets output
// row ho through filter tap r only if h + pad - r = stride*ho, i.e. r = r0 + stride*t with
// r0 = (a + pad) mod stride, and then ho = i + q0 - t with q0 = (a + pad) div stride.  The pixels of
// one residue class (a, b) of (h, w) therefore see a unit-stride correlation of the gradient with
// the sub-grid (r0 + stride_h*t, s0 + stride_w*u) of the filter's taps, so the phases together do
// exactly the products of the forward pass, none of them with an inserted zero.
struct Phase {
    int64_t n;   // pixels of the class along this axis
    int64_t t;   // taps of the class (0: these pixels receive no gradient)
    int64_t r0;  // first tap
    int64_t pad; // padding of the unit-stride gather, t - 1 - q0 (may be negative)
};

Phase make_phase(int64_t a, int64_t size, int64_t k, int64_t stride, int64_t pad) {
    Phase f;
    f.n = a < size ? (size - a + stride - 1) / stride : 0;
    f.r0 = (a + pad) % stride;
    f.t = f.r0 < k ? (k - f.r0 + stride - 1) / stride : 0;
    f.pad = f.t - 1 - (a + pad) / stride;
    return f;
}

const int64_t MAX_PHASES = 64;

// True when the strided input gradient can run phase by phase on the 32-channel gather.
bool dgrad_phased_ok(const cg_conv2d_desc* d, const void* const* in) {
    return (d->stride_h != 1 || d->stride_w != 1) && d->stride_h * d->stride_w <= MAX_PHASES &&
           all_aligned16(in, 4) && d->Cout % 32 == 0;
}

// Plan of phase (a, b); *empty is set when the class has no pixels or no taps.
cg_status plan_conv2d_dgrad_phase(const uint64_t* g_i, const uint64_t* g_ip1, const uint64_t* w_i,
                                  const uint64_t* w_ip1, uint64_t* dx_i, const cg_conv2d_desc* d,
                                  const ConvDims& cd, int64_t a, int64_t b, Plan* out, bool* empty) {
    const Phase fh = make_phase(a, d->H, d->kh, d->stride_h, d->pad_h);
    const Phase fw = make_phase(b, d->W, d->kw, d->stride_w, d->pad_w);
    *empty = fh.n == 0 || fw.n == 0 || fh.t == 0 || fw.t == 0;
    if (*empty) return CG_OK;
    const int64_t hw = fh.n * fw.n;
    const int64_t Mg = d->B * hw, Kg = fh.t * fw.t * d->Cout;
    const int64_t g_img = cd.howo * d->Cout;
    if (Mg > MAX_DIM || d->Cin > MAX_DIM || Kg > MAX_ROW_WORDS || g_img > ((int64_t)1 << 27) ||
        fh.pad > 32767 || fw.pad > 32767 || fh.pad < -32767 || fw.pad < -32767 || d->kh > 32767 || d->kw > 32767 ||
        d->kh * d->kw * d->Cin > ((int64_t)1 << 22) || d->B * d->H * d->W > MAX_DIM || fh.t * fw.t > cg::MAX_MASK_TAPS)
        return CG_ERR_UNSUPPORTED;
    const int64_t span_imgs = (cg::MAX_TILE_ROWS - 1) / hw + 2;
    if ((span_imgs < d->B ? span_imgs : d->B) * g_img * 8 > MAX_VIEW_BYTES) return CG_ERR_UNSUPPORTED;

    Plan pl = {};
    cg::GemmParams& p = pl.p;
    p.x_a = g_i; p.x_b = g_ip1; p.w_a = w_i; p.w_b = w_ip1; p.z = dx_i;
    p.M = (int)Mg; p.N = (int)d->Cin; p.K = (int)Kg;
    p.x_elems = (u64)cd.z_el;
    p.w_elems = (u64)cd.w_el;
    p.img_elems = (u64)g_img;
    p.H = (int)cd.Ho; p.W = (int)cd.Wo; p.Cin = (int)d->Cout; p.Ho = (int)fh.n; p.Wo = (int)fw.n;
    p.kh = (int)fh.t; p.kw = (int)fw.t; p.sh = 1; p.sw = 1;
    p.ph = (int)fh.pad; p.pw = (int)fw.pad;
    p.div_cin = cg::make_fast_div((uint32_t)d->Cout);
    p.div_kw = cg::make_fast_div((uint32_t)fw.t);
    p.flt_kh = (int)d->kh; p.flt_kw = (int)d->kw; p.flt_r0 = (int)fh.r0; p.flt_s0 = (int)fw.r0;
    p.flt_sh = (int)d->stride_h; p.flt_sw = (int)d->stride_w;
    p.out_H = (int)d->H; p.out_W = (int)d->W; p.out_h0 = (int)a; p.out_w0 = (int)b;
    p.out_sh = (int)d->stride_h; p.out_sw = (int)d->stride_w;
    p.div_howo = cg::make_fast_div((uint32_t)hw);
    p.div_wo = cg::make_fast_div((uint32_t)fw.n);
    p.z_prezeroed = 1;
    pl.amode = cg::A_CONV_C32; pl.bmode = cg::B_FLIP_C32;
    pl.x_bytes = (u64)cd.z_el * 8; pl.w_bytes = (u64)cd.w_el * 8; pl.z_bytes = (u64)cd.x_el * 8;
    *out = pl;
    return CG_OK;
}

// Weight gradient: DW [Cout, kh*kw*Cin] = G^T [Cout, pixels] x patches [pixels, kh*kw*Cin].  The
// gradient [pixels, Cout] is the left operand stored transposed; the right operand gathers the
// patch entries from the layer input, one K slice (32 output pixels) at a time.
cg_status plan_conv2d_wgrad(const uint64_t* g_i, const uint64_t* g_ip1, const uint64_t* x_i, const uint64_t* x_ip1,
                            uint64_t* dw_i, const cg_conv2d_desc* d, Plan* out) {
    if (!d || !g_i || !g_ip1 || !x_i || !x_ip1 || !dw_i) return CG_ERR_NULL;
    ConvDims cd;
    if (cg_status st = conv_dims(d, &cd)) return st;
    if (cg_status st = check_product_ptrs(g_i, g_ip1, x_i, x_ip1, dw_i, (u64)cd.z_el * 8, (u64)cd.x_el * 8,
                                          (u64)cd.w_el * 8))
        return st;
    // pixels are the contraction index here; slices are rebased one by one, so K may be long
    if (cd.M > ((int64_t)1 << 30) || cd.K > MAX_DIM || d->Cout > ((int64_t)1 << 22) || cd.img > ((int64_t)1 << 27) ||
        d->pad_h > 32767 || d->pad_w > 32767 || d->stride_h > 32767 || d->stride_w > 32767 ||
        d->kh > 32767 || d->kw > 32767)
        return CG_ERR_UNSUPPORTED;

    const bool pointwise = d->kh == 1 && d->kw == 1 && d->stride_h == 1 && d->stride_w == 1 &&
                           d->pad_h == 0 && d->pad_w == 0;
    if (pointwise && cd.M <= MAX_ROW_WORDS && d->Cin <= ((int64_t)1 << 22))
        // DW [Cout, Cin] = G^T x X with both operands stored [pixels, .]
        return plan_matmul(g_i, g_ip1, x_i, x_ip1, dw_i, d->Cout, d->Cin, cd.M, true, out, true, true);

    // a slice of 32 pixels touches at most this many consecutive images of the input
    const int64_t span_imgs = 31 / cd.howo + 2;
    if ((span_imgs < d->B ? span_imgs : d->B) * cd.img * 8 > MAX_VIEW_BYTES) return CG_ERR_UNSUPPORTED;

    Plan pl = {};
    cg::GemmParams& p = pl.p;
    p.x_a = g_i; p.x_b = g_ip1; p.w_a = x_i; p.w_b = x_ip1; p.z = dw_i;
    p.M = (int)d->Cout; p.N = (int)cd.K; p.K = (int)cd.M;
    p.x_elems = (u64)cd.z_el;
    p.w_elems = (u64)cd.x_el;
    p.img_elems = (u64)cd.img;
    p.H = (int)d->H; p.W = (int)d->W; p.Cin = (int)d->Cin; p.Ho = (int)cd.Ho; p.Wo = (int)cd.Wo;
    p.kh = (int)d->kh; p.kw = (int)d->kw; p.sh = (int)d->stride_h; p.sw = (int)d->stride_w;
    p.ph = (int)d->pad_h; p.pw = (int)d->pad_w;
    p.div_cin = cg::make_fast_div((uint32_t)d->Cin);
    p.div_kw = cg::make_fast_div((uint32_t)d->kw);
    p.div_howo = cg::make_fast_div((uint32_t)cd.howo);
    p.div_wo = cg::make_fast_div((uint32_t)cd.Wo);
    pl.amode = cg::A_TRANS; pl.bmode = cg::B_PATCH_T;
    pl.x_bytes = (u64)cd.z_el * 8; pl.w_bytes = (u64)cd.x_el * 8; pl.z_bytes = (u64)cd.w_el * 8;
    // The three-term product is symmetric in its operands, so the patches may as well be the left operand
    // and the gradient the right one, with DW written transposed.  Taken when that covers [Cout, kh*kw*Cin]
    // with fewer 128 x 64 tiles: a layer of up to 64 output channels then fills its tiles.
    const int64_t tiles_plain = ((d->Cout + 127) / 128) * ((cd.K + 63) / 64);
    const int64_t tiles_swapped = ((cd.K + 127) / 128) * ((d->Cout + 63) / 64);
    if (tiles_swapped < tiles_plain) {
        p.x_a = x_i; p.x_b = x_ip1; p.w_a = g_i; p.w_b = g_ip1;
        p.M = (int)cd.K; p.N = (int)d->Cout;
        p.x_elems = (u64)cd.x_el;
        p.w_elems = (u64)cd.z_el;
        pl.amode = cg::A_PATCH_T; pl.bmode = cg::B_TRANS;
        pl.x_bytes = (u64)cd.x_el * 8; pl.w_bytes = (u64)cd.z_el * 8;
    }
    *out = pl;
    return CG_OK;
}

cg_status run_direct(const Plan& pl, void* stream) {
    const hipError_t e = cg::launch_share_gemm(pl.p, pl.amode, pl.bmode, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CG_OK : CG_ERR_DEVICE;
}

// Digit-plane route: four conversions into the caller's scratch memory, then the contraction.
cg_status run_planes(Plan& pl, void* workspace, size_t workspace_bytes, void* stream) {
    if (!workspace) return CG_ERR_NULL;
    if (!aligned(workspace, 16)) return CG_ERR_ALIGN;
    const u64 need = plan_workspace_bytes(pl);
    if (workspace_bytes < need) return CG_ERR_WORKSPACE;
    const cg::GemmParams& q = pl.p;
    if (overlap(workspace, need, q.x_a, pl.x_bytes) || overlap(workspace, need, q.x_b, pl.x_bytes) ||
        overlap(workspace, need, q.w_a, pl.w_bytes) || overlap(workspace, need, q.w_b, pl.w_bytes) ||
        overlap(workspace, need, q.z, pl.z_bytes))
        return CG_ERR_ALIAS;
    char* ws = static_cast<char*>(workspace);
    char* xp_a = ws;
    char* xp_b = xp_a + round_up(pl.xp_bytes, 256);
    char* wp_sum = xp_b + round_up(pl.xp_bytes, 256);
    char* wp_a = wp_sum + round_up(pl.wp_bytes, 256);
    hipStream_t s = static_cast<hipStream_t>(stream);
    pl.p.xp_a = xp_a; pl.p.xp_b = xp_b; pl.p.wp_sum = wp_sum; pl.p.wp_a = wp_a;
    pl.p.xp_bytes = pl.xp_bytes;
    pl.p.wp_bytes = pl.wp_bytes;
    hipError_t e = cg::launch_to_planes(pl.p, pl.x_rows, pl.x_k, s);
    if (e != hipSuccess) return CG_ERR_DEVICE;
    e = cg::launch_share_gemm(pl.p, pl.planes_conv ? cg::A_PLANES_CONV : cg::A_PLANES, cg::B_PLANES, s);
    return e == hipSuccess ? CG_OK : CG_ERR_DEVICE;
}

}  // namespace

extern "C" {

cg_status cg_share_matmul(const uint64_t* x_i, const uint64_t* x_ip1, const uint64_t* y_i,
                          const uint64_t* y_ip1, uint64_t* z_i, int64_t M, int64_t N, int64_t K,
                          void* stream) {
    Plan pl;
    if (cg_status st = plan_matmul(x_i, x_ip1, y_i, y_ip1, z_i, M, N, K, true, &pl)) return st;
    return run_direct(pl, stream);
}

cg_status cg_share_matmul_acc(const uint64_t* x_i, const uint64_t* x_ip1, const uint64_t* y_i,
                              const uint64_t* y_ip1, uint64_t* z_i, int64_t M, int64_t N, int64_t K,
                              void* stream) {
    Plan pl;
    if (cg_status st = plan_matmul(x_i, x_ip1, y_i, y_ip1, z_i, M, N, K, true, &pl)) return st;
    pl.p.z_add = 1;
    return run_direct(pl, stream);
}

cg_status cg_share_conv2d_acc(const uint64_t* x_i, const uint64_t* x_ip1, const uint64_t* w_i,
                              const uint64_t* w_ip1, uint64_t* z_i, const cg_conv2d_desc* d, void* stream) {
    Plan pl;
    if (cg_status st = plan_conv2d(x_i, x_ip1, w_i, w_ip1, z_i, d, true, &pl)) return st;
    pl.p.z_add = 1;
    return run_direct(pl, stream);
}

cg_status cg_share_matmul_f64limb(const uint64_t* x_i, const uint64_t* x_ip1, const uint64_t* y_i,
                                  const uint64_t* y_ip1, uint64_t* z_i, int64_t M, int64_t N, int64_t K,
                                  void* stream) {
    Plan pl;  // validation and limits of the plain product with rows a buffer view addresses
    if (cg_status st = plan_matmul(x_i, x_ip1, y_i, y_ip1, z_i, M, N, K, true, &pl)) return st;
    if (K > MAX_ROW_WORDS) return CG_ERR_UNSUPPORTED;
    const hipError_t e = cg::launch_share_gemm_f64limb(x_i, x_ip1, y_i, y_ip1, z_i, (int)M, (int)N, (int)K,
                                                       static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CG_OK : CG_ERR_DEVICE;
}

cg_status cg_share_matmul_t(const uint64_t* x_i, const uint64_t* x_ip1, const uint64_t* y_i,
                            const uint64_t* y_ip1, uint64_t* z_i, int64_t M, int64_t N, int64_t K,
                            int trans_x, int trans_y, void* stream) {
    if ((trans_x != 0 && trans_x != 1) || (trans_y != 0 && trans_y != 1)) return CG_ERR_SHAPE;
    Plan pl;
    if (cg_status st = plan_matmul(x_i, x_ip1, y_i, y_ip1, z_i, M, N, K, true, &pl, trans_x, trans_y)) return st;
    return run_direct(pl, stream);
}

size_t cg_share_matmul_workspace_bytes(int64_t M, int64_t N, int64_t K) {
    Plan pl;
    if (plan_matmul(nullptr, nullptr, nullptr, nullptr, nullptr, M, N, K, false, &pl) != CG_OK) return 0;
    return (size_t)plan_workspace_bytes(pl);
}

cg_status cg_share_matmul_ws(const uint64_t* x_i, const uint64_t* x_ip1, const uint64_t* y_i,
                             const uint64_t* y_ip1, uint64_t* z_i, int64_t M, int64_t N, int64_t K,
                             void* workspace, size_t workspace_bytes, void* stream) {
    Plan pl;
    if (cg_status st = plan_matmul(x_i, x_ip1, y_i, y_ip1, z_i, M, N, K, true, &pl)) return st;
    if (!pl.planes_ok) return run_direct(pl, stream);
    return run_planes(pl, workspace, workspace_bytes, stream);
}

}  // extern "C"

// Scratch memory of cg_share_matmul_static: a fixed array in the library's own device image, so that
// the call never allocates.  Every GPU that loads the library holds its own copy at its own address;
// on the host the array's name is only a handle for hipGetSymbolAddress, never an address to pass on.
static __device__ __align__(256) unsigned char scratch[CG_STATIC_SCRATCH_BYTES];

namespace {

const int MAX_DEVICES = 64;
void* scratch_ptr[MAX_DEVICES];   // device address of `scratch` on device d, once looked up
std::mutex scratch_mutex;

// Device address of the current device's copy of `scratch` (looked up on the first call per device).
cg_status static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return CG_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return CG_ERR_DEVICE;
        scratch_ptr[dev] = ptr;
    }
    *out = scratch_ptr[dev];
    return CG_OK;
}

}  // namespace

extern "C" {

cg_status cg_share_matmul_static(const uint64_t* x_i, const uint64_t* x_ip1, const uint64_t* y_i,
                                 const uint64_t* y_ip1, uint64_t* z_i, int64_t M, int64_t N, int64_t K,
                                 void* stream) {
    Plan pl;
    if (cg_status st = plan_matmul(x_i, x_ip1, y_i, y_ip1, z_i, M, N, K, true, &pl)) return st;
    if (!pl.planes_ok) return run_direct(pl, stream);
    if (plan_workspace_bytes(pl) > (u64)CG_STATIC_SCRATCH_BYTES) return CG_ERR_WORKSPACE;
    void* ptr = nullptr;
    if (cg_status st = static_scratch(&ptr)) return st;
    return run_planes(pl, ptr, (size_t)CG_STATIC_SCRATCH_BYTES, stream);
}

cg_status cg_share_conv2d(const uint64_t* x_i, const uint64_t* x_ip1, const uint64_t* w_i,
                          const uint64_t* w_ip1, uint64_t* z_i, const cg_conv2d_desc* d, void* stream) {
    Plan pl;
    if (cg_status st = plan_conv2d(x_i, x_ip1, w_i, w_ip1, z_i, d, true, &pl)) return st;
    return run_direct(pl, stream);
}

int cg_share_matmul_prefers_workspace(int64_t M, int64_t N, int64_t K) {
    Plan pl;
    if (plan_matmul(nullptr, nullptr, nullptr, nullptr, nullptr, M, N, K, false, &pl) != CG_OK) return 0;
    return planes_pay(pl) ? 1 : 0;
}

int cg_share_conv2d_prefers_workspace(const cg_conv2d_desc* d) {
    Plan pl;
    if (plan_conv2d(nullptr, nullptr, nullptr, nullptr, nullptr, d, false, &pl) != CG_OK) return 0;
    return planes_pay(pl) ? 1 : 0;
}

size_t cg_share_conv2d_workspace_bytes(const cg_conv2d_desc* d) {
    Plan pl;
    if (plan_conv2d(nullptr, nullptr, nullptr, nullptr, nullptr, d, false, &pl) != CG_OK) return 0;
    return (size_t)plan_workspace_bytes(pl);
}

cg_status cg_share_conv2d_ws(const uint64_t* x_i, const uint64_t* x_ip1, const uint64_t* w_i,
                             const uint64_t* w_ip1, uint64_t* z_i, const cg_conv2d_desc* d,
                             void* workspace, size_t workspace_bytes, void* stream) {
    Plan pl;
    if (cg_status st = plan_conv2d(x_i, x_ip1, w_i, w_ip1, z_i, d, true, &pl)) return st;
    if (!pl.planes_ok) return run_direct(pl, stream);
    return run_planes(pl, workspace, workspace_bytes, stream);
}

cg_status cg_share_conv2d_dgrad(const uint64_t* g_i, const uint64_t* g_ip1, const uint64_t* w_i,
                                const uint64_t* w_ip1, uint64_t* dx_i, const cg_conv2d_desc* d, void* stream) {
    Plan pl;
    const cg_status generic = plan_conv2d_dgrad(g_i, g_ip1, w_i, w_ip1, dx_i, d, &pl);
    if (generic != CG_OK && generic != CG_ERR_UNSUPPORTED) return generic;  // arguments are wrong either way
    auto fallback = [&]() { return generic == CG_OK ? run_direct(pl, stream) : generic; };
    const void* in[4] = {g_i, g_ip1, w_i, w_ip1};
    if (!dgrad_phased_ok(d, in)) return fallback();
    // strided, 32-channel gather: one unit-stride product per residue class of the input pixels.  All
    // phases are planned before the first launch, so that an unsupported one leaves dx untouched and
    // the whole call falls back to the zero-interleaved gather.
    ConvDims cd;
    if (cg_status st = conv_dims(d, &cd)) return st;
    Plan phase[MAX_PHASES];
    bool empty[MAX_PHASES];
    int n = 0;
    for (int64_t a = 0; a < d->stride_h; ++a)
        for (int64_t b = 0; b < d->stride_w; ++b, ++n)
            if (plan_conv2d_dgrad_phase(g_i, g_ip1, w_i, w_ip1, dx_i, d, cd, a, b, &phase[n], &empty[n]) != CG_OK)
                return fallback();
    // pixels of classes without taps keep the zeros; launches that split K add into them
    if (cg::launch_zero_words(dx_i, (size_t)cd.x_el, static_cast<hipStream_t>(stream)) != hipSuccess)
        return CG_ERR_DEVICE;
    for (int i = 0; i < n; ++i)
        if (!empty[i])
            if (cg_status st = run_direct(phase[i], stream)) return st;
    return CG_OK;
}

cg_status cg_share_conv2d_wgrad(const uint64_t* g_i, const uint64_t* g_ip1, const uint64_t* x_i,
                                const uint64_t* x_ip1, uint64_t* dw_i, const cg_conv2d_desc* d, void* stream) {
    Plan pl;
    if (cg_status st = plan_conv2d_wgrad(g_i, g_ip1, x_i, x_ip1, dw_i, d, &pl)) return st;
    return run_direct(pl, stream);
}

cg_status cg_share_add(const uint64_t* xa, const uint64_t* xb, const uint64_t* ya, const uint64_t* yb,
                       uint64_t* za, uint64_t* zb, size_t n, void* stream) {
    if (n == 0) return CG_OK;  // nothing to do: pointers are not looked at
    const void* ptrs[6] = {xa, xb, ya, yb, za, zb};
    if (cg_status st = check_ptrs(ptrs, 6)) return st;
    if (n > (SIZE_MAX >> 4)) return CG_ERR_SHAPE;
    const u64 bytes = (u64)n * 8;
    for (int o = 4; o < 6; ++o)
        for (int i = 0; i < 4; ++i)
            if (bad_overlap(ptrs[o], ptrs[i], bytes)) return CG_ERR_ALIAS;
    if (n && overlap(za, bytes, zb, bytes)) return CG_ERR_ALIAS;
    AddOp f = {xa, xb, ya, yb, za, zb};
    return launch_ew(n, all_aligned16(ptrs, 6), f, stream);
}

cg_status cg_share_mul_public(const uint64_t* xa, const uint64_t* xb, uint64_t alpha, uint64_t* za,
                              uint64_t* zb, size_t n, void* stream) {
    if (n == 0) return CG_OK;  // nothing to do: pointers are not looked at
    const void* ptrs[4] = {xa, xb, za, zb};
    if (cg_status st = check_ptrs(ptrs, 4)) return st;
    if (n > (SIZE_MAX >> 4)) return CG_ERR_SHAPE;
    const u64 bytes = (u64)n * 8;
    for (int o = 2; o < 4; ++o)
        for (int i = 0; i < 2; ++i)
            if (bad_overlap(ptrs[o], ptrs[i], bytes)) return CG_ERR_ALIAS;
    if (n && overlap(za, bytes, zb, bytes)) return CG_ERR_ALIAS;
    MulPublicOp f = {xa, xb, alpha, za, zb};
    return launch_ew(n, all_aligned16(ptrs, 4), f, stream);
}

cg_status cg_share_add_public(const uint64_t* xa, const uint64_t* xb, uint64_t gamma, int party,
                              uint64_t* za, uint64_t* zb, size_t n, void* stream) {
    if (n == 0) return CG_OK;  // nothing to do: pointers are not looked at
    const void* ptrs[4] = {xa, xb, za, zb};
    if (cg_status st = check_ptrs(ptrs, 4)) return st;
    if (party < 0 || party > 2 || n > (SIZE_MAX >> 4)) return CG_ERR_SHAPE;
    const u64 bytes = (u64)n * 8;
    for (int o = 2; o < 4; ++o)
        for (int i = 0; i < 2; ++i)
            if (bad_overlap(ptrs[o], ptrs[i], bytes)) return CG_ERR_ALIAS;
    if (n && overlap(za, bytes, zb, bytes)) return CG_ERR_ALIAS;
    // share index 0 is the first component of party 0 and the second component of party 2
    AddPublicOp f = {xa, xb, party == 0 ? gamma : 0, party == 2 ? gamma : 0, za, zb};
    return launch_ew(n, all_aligned16(ptrs, 4), f, stream);
}

cg_status cg_share_mul(const uint64_t* x_i, const uint64_t* x_ip1, const uint64_t* y_i, const uint64_t* y_ip1,
                       uint64_t* z_i, size_t n, size_t period, void* stream) {
    if (n == 0) return CG_OK;
    const void* ptrs[5] = {x_i, x_ip1, y_i, y_ip1, z_i};
    if (cg_status st = check_ptrs(ptrs, 5)) return st;
    if (period == 0 || period > n || n % period != 0 || n > (SIZE_MAX >> 4)) return CG_ERR_SHAPE;
    const u64 bytes = (u64)n * 8, ybytes = (u64)period * 8;
    if (bad_overlap(z_i, x_i, bytes) || bad_overlap(z_i, x_ip1, bytes)) return CG_ERR_ALIAS;
    if (overlap(z_i, bytes, y_i, ybytes) || overlap(z_i, bytes, y_ip1, ybytes)) {
        // in place over y is only sound when y is not broadcast and the pointers coincide
        if (!(period == n && (z_i == y_i || z_i == y_ip1) && !bad_overlap(z_i, y_i, bytes) &&
              !bad_overlap(z_i, y_ip1, bytes)))
            return CG_ERR_ALIAS;
    }
    PartyMulOp f = {x_i, x_ip1, y_i, y_ip1, z_i, period};
    const bool vec = all_aligned16(ptrs, 5) && period % 2 == 0;
    return launch_ew(n, vec, f, stream);
}

cg_status cg_share_bias_add(const uint64_t* xa, const uint64_t* xb, const uint64_t* ba, const uint64_t* bb,
                            uint64_t* za, uint64_t* zb, size_t n, size_t period, void* stream) {
    if (n == 0) return CG_OK;
    const void* ptrs[6] = {xa, xb, ba, bb, za, zb};
    if (cg_status st = check_ptrs(ptrs, 6)) return st;
    if (period == 0 || period > n || n % period != 0 || n > (SIZE_MAX >> 4)) return CG_ERR_SHAPE;
    const u64 bytes = (u64)n * 8, bbytes = (u64)period * 8;
    if (bad_overlap(za, xa, bytes) || bad_overlap(za, xb, bytes) || bad_overlap(zb, xa, bytes) ||
        bad_overlap(zb, xb, bytes) || overlap(za, bytes, zb, bytes))
        return CG_ERR_ALIAS;
    if (overlap(za, bytes, ba, bbytes) || overlap(za, bytes, bb, bbytes) || overlap(zb, bytes, ba, bbytes) ||
        overlap(zb, bytes, bb, bbytes))
        return CG_ERR_ALIAS;
    BiasAddOp f = {xa, xb, ba, bb, za, zb, period};
    return launch_ew(n, all_aligned16(ptrs, 6) && period % 2 == 0, f, stream);
}

cg_status cg_share_col_sum(const uint64_t* xa, const uint64_t* xb, uint64_t* za, uint64_t* zb, size_t rows,
                           size_t cols, void* stream) {
    if (cols == 0) return CG_OK;
    if (!za || !zb) return CG_ERR_NULL;
    if (!aligned(za, 8) || !aligned(zb, 8)) return CG_ERR_ALIGN;
    size_t n;
    if (__builtin_mul_overflow(rows, cols, &n) || n > (SIZE_MAX >> 4)) return CG_ERR_SHAPE;
    if (overlap(za, (u64)cols * 8, zb, (u64)cols * 8)) return CG_ERR_ALIAS;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (rows > 0) {
        if (!xa || !xb) return CG_ERR_NULL;
        if (!aligned(xa, 8) || !aligned(xb, 8)) return CG_ERR_ALIGN;
        const u64 xbytes = (u64)n * 8, zbytes = (u64)cols * 8;
        if (overlap(za, zbytes, xa, xbytes) || overlap(za, zbytes, xb, xbytes) || overlap(zb, zbytes, xa, xbytes) ||
            overlap(zb, zbytes, xb, xbytes))
            return CG_ERR_ALIAS;
    }
    const size_t col_tiles = (cols + 63) / 64;
    if (rows > 0 && col_tiles > 0x7FFFFFFF) return CG_ERR_UNSUPPORTED;  // before anything is launched
    size_t zblocks = (cols + 255) / 256;
    if (zblocks > 1024) zblocks = 1024;
    hipLaunchKernelGGL(zero2_kernel, dim3((unsigned)zblocks), dim3(256), 0, s, za, zb, cols);
    if (rows > 0) {
        // about eight blocks per compute unit, at least 16 rows per wave
        size_t row_blocks = (2048 + col_tiles - 1) / col_tiles;
        const size_t max_rb = (rows + 63) / 64;
        if (row_blocks > max_rb) row_blocks = max_rb;
        if (row_blocks < 1) row_blocks = 1;
        if (row_blocks > 65535) row_blocks = 65535;
        hipLaunchKernelGGL(col_sum_kernel, dim3((unsigned)col_tiles, (unsigned)row_blocks), dim3(256), 0, s, xa, xb, za,
                           zb, rows, cols);
    }
    return hipGetLastError() == hipSuccess ? CG_OK : CG_ERR_DEVICE;
}

cg_status cg_share_sum_pool2d(const uint64_t* xa, const uint64_t* xb, uint64_t* za, uint64_t* zb,
                              const cg_pool2d_desc* d, void* stream) {
    if (!xa || !xb || !za || !zb || !d) return CG_ERR_NULL;
    if (d->B < 1 || d->H < 1 || d->W < 1 || d->C < 1 || d->kh < 1 || d->kw < 1 || d->stride_h < 1 ||
        d->stride_w < 1 || d->pad_h < 0 || d->pad_w < 0)
        return CG_ERR_SHAPE;
    const int64_t LIM = 0x7FFFFFFF;
    if (d->B > LIM || d->H > LIM || d->W > LIM || d->C > LIM || d->kh > LIM || d->kw > LIM ||
        d->stride_h > LIM || d->stride_w > LIM || d->pad_h > LIM || d->pad_w > LIM)
        return CG_ERR_UNSUPPORTED;
    const int64_t span_h = d->H + 2 * d->pad_h - d->kh, span_w = d->W + 2 * d->pad_w - d->kw;
    if (span_h < 0 || span_w < 0) return CG_ERR_SHAPE;
    const int64_t Ho = span_h / d->stride_h + 1, Wo = span_w / d->stride_w + 1;
    int64_t x_el, z_el, tmp;
    if (mul_overflows(d->B, d->H, &tmp) || mul_overflows(tmp, d->W, &tmp) || mul_overflows(tmp, d->C, &x_el) ||
        mul_overflows(d->B, Ho, &tmp) || mul_overflows(tmp, Wo, &tmp) || mul_overflows(tmp, d->C, &z_el) ||
        mul_overflows(x_el, 8, &tmp) || mul_overflows(z_el, 8, &tmp))
        return CG_ERR_SHAPE;
    const void* ptrs[4] = {xa, xb, za, zb};
    if (cg_status st = check_ptrs(ptrs, 4)) return st;
    const u64 xb_ = (u64)x_el * 8, zb_ = (u64)z_el * 8;
    if (overlap(za, zb_, xa, xb_) || overlap(za, zb_, xb, xb_) || overlap(zb, zb_, xa, xb_) ||
        overlap(zb, zb_, xb, xb_) || overlap(za, zb_, zb, zb_))
        return CG_ERR_ALIAS;
    const int vec = (d->C % 2 == 0) && all_aligned16(ptrs, 4);
    const size_t total = (size_t)z_el / (vec ? 2 : 1);
    size_t blocks = (total + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(sum_pool_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream), xa, xb,
                       za, zb, (int)d->B, (int)d->H, (int)d->W, (int)d->C, (int)Ho, (int)Wo, (int)d->kh, (int)d->kw,
                       (int)d->stride_h, (int)d->stride_w, (int)d->pad_h, (int)d->pad_w, vec);
    return hipGetLastError() == hipSuccess ? CG_OK : CG_ERR_DEVICE;
}

cg_status cg_zero_share(const uint8_t* key_self, const uint8_t* key_prev, uint64_t nonce, uint64_t first,
                        uint64_t* alpha, size_t n, void* stream) {
    if (!key_self || !key_prev) return CG_ERR_NULL;
    if (n == 0) return CG_OK;
    if (!alpha) return CG_ERR_NULL;
    if (!aligned(alpha, 8)) return CG_ERR_ALIGN;
    if (n > (SIZE_MAX >> 4) || first + n < first) return CG_ERR_SHAPE;
    const hipError_t e = cg::launch_zero_share(nullptr, alpha, n, key_self, key_prev, nonce, first,
                                               static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CG_OK : CG_ERR_DEVICE;
}

cg_status cg_reshare(const uint64_t* z_i, const uint8_t* key_self, const uint8_t* key_prev, uint64_t nonce,
                     uint64_t first, uint64_t* out, size_t n, void* stream) {
    if (!key_self || !key_prev) return CG_ERR_NULL;
    if (n == 0) return CG_OK;
    if (!z_i || !out) return CG_ERR_NULL;
    if (!aligned(z_i, 8) || !aligned(out, 8)) return CG_ERR_ALIGN;
    if (n > (SIZE_MAX >> 4) || first + n < first) return CG_ERR_SHAPE;
    if (bad_overlap(out, z_i, (u64)n * 8)) return CG_ERR_ALIAS;
    const hipError_t e = cg::launch_zero_share(z_i, out, n, key_self, key_prev, nonce, first,
                                               static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CG_OK : CG_ERR_DEVICE;
}

cg_status cg_bshare_xor(const uint64_t* xa, const uint64_t* xb, const uint64_t* ya, const uint64_t* yb,
                        uint64_t* za, uint64_t* zb, size_t n, void* stream) {
    if (n == 0) return CG_OK;
    const void* ptrs[6] = {xa, xb, ya, yb, za, zb};
    if (cg_status st = check_ptrs(ptrs, 6)) return st;
    if (n > (SIZE_MAX >> 4)) return CG_ERR_SHAPE;
    const u64 bytes = (u64)n * 8;
    for (int o = 4; o < 6; ++o)
        for (int i = 0; i < 4; ++i)
            if (bad_overlap(ptrs[o], ptrs[i], bytes)) return CG_ERR_ALIAS;
    if (overlap(za, bytes, zb, bytes)) return CG_ERR_ALIAS;
    BXorOp f = {xa, xb, ya, yb, za, zb};
    return launch_ew(n, all_aligned16(ptrs, 6), f, stream);
}

cg_status cg_bshare_and(const uint64_t* x_i, const uint64_t* x_ip1, const uint64_t* y_i, const uint64_t* y_ip1,
                        uint64_t* z_i, size_t n, void* stream) {
    if (n == 0) return CG_OK;
    const void* ptrs[5] = {x_i, x_ip1, y_i, y_ip1, z_i};
    if (cg_status st = check_ptrs(ptrs, 5)) return st;
    if (n > (SIZE_MAX >> 4)) return CG_ERR_SHAPE;
    const u64 bytes = (u64)n * 8;
    for (int i = 0; i < 4; ++i)
        if (bad_overlap(z_i, ptrs[i], bytes)) return CG_ERR_ALIAS;
    BAndOp f = {x_i, x_ip1, y_i, y_ip1, z_i};
    return launch_ew(n, all_aligned16(ptrs, 5), f, stream);
}

cg_status cg_bshare_prefix_stage(const uint64_t* p_i, const uint64_t* p_ip1, const uint64_t* g_i,
                                 const uint64_t* g_ip1, int shift, uint64_t* p_out, uint64_t* g_out, size_t n,
                                 void* stream) {
    if (shift < 1 || shift > 63) return CG_ERR_SHAPE;
    if (n == 0) return CG_OK;
    const void* in[5] = {p_i, p_ip1, g_i, g_ip1, g_out};
    if (cg_status st = check_ptrs(in, 5)) return st;
    if (p_out && !aligned(p_out, 8)) return CG_ERR_ALIGN;
    if (n > (SIZE_MAX >> 4)) return CG_ERR_SHAPE;
    const u64 bytes = (u64)n * 8;
    // every output element depends only on the same element of the inputs, so in place is fine;
    // partial overlaps and coinciding outputs are not
    for (int i = 0; i < 4; ++i)
        if (bad_overlap(g_out, in[i], bytes) || (p_out && bad_overlap(p_out, in[i], bytes))) return CG_ERR_ALIAS;
    if (p_out && overlap(p_out, bytes, g_out, bytes)) return CG_ERR_ALIAS;
    PrefixStageOp f = {p_i, p_ip1, g_i, g_ip1, p_out, g_out, shift};
    const void* all[6] = {p_i, p_ip1, g_i, g_ip1, g_out, p_out ? p_out : g_out};
    return launch_ew(n, all_aligned16(all, 6), f, stream);
}

cg_status cg_bshare_csa(const uint64_t* a_i, const uint64_t* a_ip1, const uint64_t* b_i, const uint64_t* b_ip1,
                        const uint64_t* c_i, const uint64_t* c_ip1, uint64_t* s_i, uint64_t* s_ip1, uint64_t* carry_i,
                        size_t n, void* stream) {
    if (n == 0) return CG_OK;
    const void* ptrs[9] = {a_i, a_ip1, b_i, b_ip1, c_i, c_ip1, s_i, s_ip1, carry_i};
    if (cg_status st = check_ptrs(ptrs + 6, 3)) return st;  // outputs
    for (int i = 0; i < 6; ++i)                               // inputs: null stands for an all-zero component
        if (ptrs[i] && !aligned(ptrs[i], 8)) return CG_ERR_ALIGN;
    if (n > (SIZE_MAX >> 4)) return CG_ERR_SHAPE;
    const u64 bytes = (u64)n * 8;
    for (int o = 6; o < 9; ++o) {
        for (int i = 0; i < 6; ++i)
            if (ptrs[i] && bad_overlap(ptrs[o], ptrs[i], bytes)) return CG_ERR_ALIAS;
        for (int o2 = o + 1; o2 < 9; ++o2)
            if (overlap(ptrs[o], bytes, ptrs[o2], bytes)) return CG_ERR_ALIAS;
    }
    CsaOp f = {a_i, a_ip1, b_i, b_ip1, c_i, c_ip1, s_i, s_ip1, carry_i};
    return launch_ew(n, all_aligned16(ptrs, 9), f, stream);
}

cg_status cg_bshare_half_adder(const uint64_t* s_i, const uint64_t* s_ip1, const uint64_t* t_i, const uint64_t* t_ip1,
                               uint64_t* p_i, uint64_t* p_ip1, uint64_t* g_i, size_t n, void* stream) {
    if (n == 0) return CG_OK;
    const void* ptrs[7] = {s_i, s_ip1, t_i, t_ip1, p_i, p_ip1, g_i};
    if (cg_status st = check_ptrs(ptrs, 7)) return st;
    if (n > (SIZE_MAX >> 4)) return CG_ERR_SHAPE;
    const u64 bytes = (u64)n * 8;
    for (int o = 4; o < 7; ++o) {
        for (int i = 0; i < 4; ++i)
            if (bad_overlap(ptrs[o], ptrs[i], bytes)) return CG_ERR_ALIAS;
        for (int o2 = o + 1; o2 < 7; ++o2)
            if (overlap(ptrs[o], bytes, ptrs[o2], bytes)) return CG_ERR_ALIAS;
    }
    HalfAdderOp f = {s_i, s_ip1, t_i, t_ip1, p_i, p_ip1, g_i};
    return launch_ew(n, all_aligned16(ptrs, 7), f, stream);
}

cg_status cg_bshare_carry_level(const uint64_t* p_i, const uint64_t* p_ip1, const uint64_t* g_i, const uint64_t* g_ip1,
                                uint64_t* p_out, uint64_t* g_out, size_t planes_out, size_t m, void* stream) {
    size_t n;
    if (__builtin_mul_overflow(planes_out, m, &n) || n > (SIZE_MAX >> 5)) return CG_ERR_SHAPE;
    if (n == 0) return CG_OK;
    const void* in[5] = {p_i, p_ip1, g_i, g_ip1, g_out};
    if (cg_status st = check_ptrs(in, 5)) return st;
    if (p_out && !aligned(p_out, 8)) return CG_ERR_ALIGN;
    const u64 in_bytes = (u64)n * 16, out_bytes = (u64)n * 8;
    // outputs are half the size of the inputs and indexed differently: no overlap with them at all
    for (int i = 0; i < 4; ++i)
        if (overlap(g_out, out_bytes, in[i], in_bytes) || (p_out && overlap(p_out, out_bytes, in[i], in_bytes)))
            return CG_ERR_ALIAS;
    if (p_out && overlap(p_out, out_bytes, g_out, out_bytes)) return CG_ERR_ALIAS;
    CarryLevelOp f = {p_i, p_ip1, g_i, g_ip1, p_out, g_out, m};
    const void* all[6] = {p_i, p_ip1, g_i, g_ip1, g_out, p_out ? p_out : g_out};
    return launch_ew(n, all_aligned16(all, 6) && m % 2 == 0, f, stream);
}

cg_status cg_bit_transpose64(const uint64_t* src, uint64_t* dst, size_t n, void* stream) {
    if (n == 0) return CG_OK;
    if (!src || !dst) return CG_ERR_NULL;
    if (!aligned(src, 8) || !aligned(dst, 8)) return CG_ERR_ALIGN;
    if (n % 64 != 0 || n > (SIZE_MAX >> 4)) return CG_ERR_SHAPE;
    if (overlap(dst, (u64)n * 8, src, (u64)n * 8)) return CG_ERR_ALIAS;
    const size_t m = n / 64;
    size_t blocks = (m + 4 * 32 - 1) / (4 * 32);   // four waves per block, 32 blocks of 64 words per wave and trip
    if (blocks > 256 * 16) blocks = 256 * 16;
    hipLaunchKernelGGL(bit_transpose_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream), src,
                       dst, m);
    return hipGetLastError() == hipSuccess ? CG_OK : CG_ERR_DEVICE;
}

cg_status cg_bits_unpack(const uint64_t* plane, uint64_t* out, size_t n, void* stream) {
    if (n == 0) return CG_OK;
    if (!plane || !out) return CG_ERR_NULL;
    if (!aligned(plane, 8) || !aligned(out, 8)) return CG_ERR_ALIGN;
    if (n > (SIZE_MAX >> 4)) return CG_ERR_SHAPE;
    if (overlap(out, (u64)n * 8, plane, (u64)((n + 63) / 64) * 8)) return CG_ERR_ALIAS;
    size_t blocks = (n + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    hipLaunchKernelGGL(bits_unpack_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream), plane,
                       out, n);
    return hipGetLastError() == hipSuccess ? CG_OK : CG_ERR_DEVICE;
}

cg_status cg_bzero_share(const uint8_t* key_self, const uint8_t* key_prev, uint64_t nonce, uint64_t first,
                         uint64_t* beta, size_t n, void* stream) {
    if (!key_self || !key_prev) return CG_ERR_NULL;
    if (n == 0) return CG_OK;
    if (!beta) return CG_ERR_NULL;
    if (!aligned(beta, 8)) return CG_ERR_ALIGN;
    if (n > (SIZE_MAX >> 4) || first + n < first) return CG_ERR_SHAPE;
    const hipError_t e = cg::launch_prf_combine(nullptr, nullptr, beta, n, key_self, key_prev, nonce, first, 0, nullptr,
                                                0, false, static_cast<hipStream_t>(stream), true);
    return e == hipSuccess ? CG_OK : CG_ERR_DEVICE;
}

cg_status cg_breshare(const uint64_t* z_i, const uint8_t* key_self, const uint8_t* key_prev, uint64_t nonce,
                      uint64_t first, uint64_t* out, size_t n, void* stream) {
    if (!key_self || !key_prev) return CG_ERR_NULL;
    if (n == 0) return CG_OK;
    if (!z_i || !out) return CG_ERR_NULL;
    if (!aligned(z_i, 8) || !aligned(out, 8)) return CG_ERR_ALIGN;
    if (n > (SIZE_MAX >> 4) || first + n < first) return CG_ERR_SHAPE;
    if (bad_overlap(out, z_i, (u64)n * 8)) return CG_ERR_ALIAS;
    const hipError_t e = cg::launch_prf_combine(z_i, nullptr, out, n, key_self, key_prev, nonce, first, 0, nullptr, 0,
                                                false, static_cast<hipStream_t>(stream), true);
    return e == hipSuccess ? CG_OK : CG_ERR_DEVICE;
}

cg_status cg_prf_words(const uint8_t* key, uint64_t nonce, uint64_t first, uint64_t* out, size_t n, void* stream) {
    if (!key) return CG_ERR_NULL;
    if (n == 0) return CG_OK;
    if (!out) return CG_ERR_NULL;
    if (!aligned(out, 8)) return CG_ERR_ALIGN;
    if (n > (SIZE_MAX >> 4) || first + n < first) return CG_ERR_SHAPE;
    const hipError_t e = cg::launch_prf_combine(nullptr, nullptr, out, n, nullptr, nullptr, 0, first, 0, key, nonce,
                                                true, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CG_OK : CG_ERR_DEVICE;
}

cg_status cg_trunc1_local(const uint64_t* z_i, const uint64_t* msg, const uint8_t* key_self, const uint8_t* key_prev,
                          uint64_t nonce, uint64_t first, int d, const uint8_t* key_mask, uint64_t mask_nonce,
                          uint64_t* out, size_t n, void* stream) {
    if (!key_self || !key_prev) return CG_ERR_NULL;
    if (d < 0 || d > 63) return CG_ERR_SHAPE;
    // a mask drawn from one of the alpha streams themselves would cancel against alpha instead of blinding
    if (key_mask && mask_nonce == nonce &&
        (memcmp(key_mask, key_self, 16) == 0 || memcmp(key_mask, key_prev, 16) == 0))
        return CG_ERR_SHAPE;
    if (n == 0) return CG_OK;
    if (!z_i || !out) return CG_ERR_NULL;
    if (!aligned(z_i, 8) || !aligned(out, 8) || (msg && !aligned(msg, 8))) return CG_ERR_ALIGN;
    if (n > (SIZE_MAX >> 4) || first + n < first) return CG_ERR_SHAPE;
    const u64 bytes = (u64)n * 8;
    if (bad_overlap(out, z_i, bytes) || (msg && bad_overlap(out, msg, bytes))) return CG_ERR_ALIAS;
    const hipError_t e = cg::launch_prf_combine(z_i, msg, out, n, key_self, key_prev, nonce, first, d, key_mask,
                                                mask_nonce, false, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CG_OK : CG_ERR_DEVICE;
}

cg_status cg_reconstruct(const uint64_t* s0, const uint64_t* s1, const uint64_t* s2, uint64_t* out,
                         size_t n, void* stream) {
    if (n == 0) return CG_OK;  // nothing to do: pointers are not looked at
    const void* ptrs[4] = {s0, s1, s2, out};
    if (cg_status st = check_ptrs(ptrs, 4)) return st;
    if (n > (SIZE_MAX >> 4)) return CG_ERR_SHAPE;
    const u64 bytes = (u64)n * 8;
    for (int i = 0; i < 3; ++i)
        if (bad_overlap(out, ptrs[i], bytes)) return CG_ERR_ALIAS;
    ReconstructOp f = {s0, s1, s2, out};
    return launch_ew(n, all_aligned16(ptrs, 4), f, stream);
}

}  // extern "C"
