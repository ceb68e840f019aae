// Zero shares from an AES-128 PRF and the reshare step z_i + alpha_i
// (CryptGPU Sec. III-B "Protocol initialization", "Multiplication"; Sec. IV
// "Pseudorandom generators on the GPU": AES is the PRF).
//
// alpha_i[j] = F(k_i, j) - F(k_{i-1}, j) mod 2^64.  F(k, j) is AES-128 in counter
// mode: input block = (block index j >> 1 as 64-bit little-endian, nonce as 64-bit
// little-endian), output word = ciphertext bytes 0..7 (j even) or 8..15 (j odd) as
// a little-endian integer.  One thread encrypts one block under both keys and
// produces two consecutive words of alpha.
//
// AES rounds use the classic 32-bit table formulation of FIPS-197: the table
// T0[x] = (2 S[x], S[x], S[x], 3 S[x]); the other three columns of the MixColumns
// matrix are its byte rotations T1 = rotl8(T0), T2 = rotl16(T0), T3 = rotl8(T2).
// Rotation distributes over XOR, so with T0 and T2 both in memory a column costs one
// rotation: (T0[a] ^ T2[c]) ^ rotl8(T0[b] ^ T2[d]).  The last round uses the S-box
// byte of T0.  Each table sits in LDS once per bank (64 copies, 64 KiB each, 128 KiB
// per block of 16 waves): lane i reads entry x of table t at byte 65536 t + 256 x + 4 i,
// always from bank i, so the data-dependent lookups of a wave never collide, and the
// whole address is ONE byte permute of (state word, lane constant).  Round keys are
// expanded on the host and passed by value.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include "prf.h"

namespace cg {

namespace {

typedef uint32_t u32;
typedef uint64_t u64;

// ---- host: tables and key schedule ------------------------------------------
// S-box via discrete logarithms to the generator 3 of GF(2^8)*, then the affine map.
struct AesTables {
    uint8_t sbox[256];
    u32 t0[256];
    AesTables() {
        uint8_t exp3[256], log3[256];
        uint8_t x = 1;
        for (int i = 0; i < 255; ++i) {
            exp3[i] = x;
            log3[x] = (uint8_t)i;
            const uint8_t x2 = (uint8_t)((x << 1) ^ ((x & 0x80) ? 0x1B : 0));  // x * 2
            x = (uint8_t)(x2 ^ x);                                             // x * 3
        }
        for (int v = 0; v < 256; ++v) {
            const uint8_t inv = v ? exp3[(255 - log3[v]) % 255] : 0;
            uint8_t s = inv;
            s ^= (uint8_t)((inv << 1) | (inv >> 7));
            s ^= (uint8_t)((inv << 2) | (inv >> 6));
            s ^= (uint8_t)((inv << 3) | (inv >> 5));
            s ^= (uint8_t)((inv << 4) | (inv >> 4));
            s ^= 0x63;
            sbox[v] = s;
            const uint8_t s2 = (uint8_t)((s << 1) ^ ((s & 0x80) ? 0x1B : 0));
            const uint8_t s3 = (uint8_t)(s2 ^ s);
            t0[v] = (u32)s2 | ((u32)s << 8) | ((u32)s << 16) | ((u32)s3 << 24);
        }
    }
};

const AesTables& tables() {
    static const AesTables t;
    return t;
}

// Round keys as 44 little-endian column words.
void expand_key(const uint8_t key[16], u32 rk[44]) {
    const uint8_t* sb = tables().sbox;
    for (int i = 0; i < 4; ++i)
        rk[i] = (u32)key[4 * i] | ((u32)key[4 * i + 1] << 8) | ((u32)key[4 * i + 2] << 16) | ((u32)key[4 * i + 3] << 24);
    u32 rcon = 1;
    for (int i = 4; i < 44; ++i) {
        u32 t = rk[i - 1];
        if ((i & 3) == 0) {
            t = (t >> 8) | (t << 24);  // RotWord on little-endian bytes
            t = (u32)sb[t & 0xFF] | ((u32)sb[(t >> 8) & 0xFF] << 8) | ((u32)sb[(t >> 16) & 0xFF] << 16) |
                ((u32)sb[t >> 24] << 24);
            t ^= rcon;
            rcon = (rcon << 1) ^ ((rcon & 0x80) ? 0x11B : 0);
        }
        rk[i] = rk[i - 4] ^ t;
    }
}

struct PrfKeys {
    u32 self[44], prev[44], mask[44];
};

// ---- device ------------------------------------------------------------------
constexpr int PRF_THREADS = 1024;

// LDS byte address of a table entry: byte 0 = 4 * (lane % 64) and byte 2 = table number
// come from the lane constant `lc` = 4 * lane | 0x0100, byte 1 = byte `B` of the state word.
// v_perm_b32(S0, S1, sel): selector values 0-3 pick bytes of S1, 4-7 bytes of S0, 0x0c gives 0.
template <int B, int TABLE>
__device__ __forceinline__ u32 lut(const char* __restrict__ tbl, u32 state, u32 lc) {
    constexpr u32 sel = 0x0C000000u | (TABLE ? 0x00010000u : 0x000C0000u) | ((u32)(4 + B) << 8);
    return *reinterpret_cast<const u32*>(tbl + __builtin_amdgcn_perm(state, lc, sel));
}

__device__ __forceinline__ u32 rotl8(u32 v) { return __builtin_amdgcn_alignbit(v, v, 24); }

// one output column of a full round: bytes 0..3 taken from state words a, b, c, d
__device__ __forceinline__ u32 column(const char* tbl, u32 lc, u32 a, u32 b, u32 c, u32 d, u32 rk) {
    return (lut<0, 0>(tbl, a, lc) ^ lut<2, 1>(tbl, c, lc)) ^ rotl8(lut<1, 0>(tbl, b, lc) ^ lut<3, 1>(tbl, d, lc)) ^ rk;
}

// one output word of the last round: S-box bytes (byte 1 of T0) of byte 0 of a, 1 of b, 2 of c, 3 of d
__device__ __forceinline__ u32 last_column(const char* tbl, u32 lc, u32 a, u32 b, u32 c, u32 d, u32 rk) {
    const u32 ta = lut<0, 0>(tbl, a, lc), tb = lut<1, 0>(tbl, b, lc), tc = lut<2, 0>(tbl, c, lc),
              td = lut<3, 0>(tbl, d, lc);
    const u32 lo = __builtin_amdgcn_perm(tb, ta, 0x0C0C0501u);  // (ta.b1, tb.b1, 0, 0)
    const u32 hi = __builtin_amdgcn_perm(td, tc, 0x0C0C0501u);
    return __builtin_amdgcn_perm(hi, lo, 0x05040100u) ^ rk;
}

// NS independent encryptions side by side, round by round.  The round loop is NOT unrolled and the round keys
// are indexed by the loop counter, so that they are fetched by scalar loads as the rounds go (one round ahead):
// keeping two or three whole key schedules in scalar registers does not fit and would be spilled into vector lanes.
template <int NS>
__device__ __forceinline__ void aes_blocks(const char* __restrict__ tbl, u32 lc, const u32* const (&rk)[NS],
                                           const u32 (&in)[NS][4], u32 (&out)[NS][4]) {
    u32 s[NS][4], k[NS][4];
#pragma unroll
    for (int e = 0; e < NS; ++e) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            s[e][c] = in[e][c] ^ rk[e][c];
            k[e][c] = rk[e][4 + c];
        }
    }
#pragma unroll 3
    for (int r = 1; r < 10; ++r) {
        u32 nk[NS][4];
#pragma unroll
        for (int e = 0; e < NS; ++e)
#pragma unroll
            for (int c = 0; c < 4; ++c) nk[e][c] = rk[e][4 * (r + 1) + c];
#pragma unroll
        for (int e = 0; e < NS; ++e) {
            const u32 n0 = column(tbl, lc, s[e][0], s[e][1], s[e][2], s[e][3], k[e][0]);
            const u32 n1 = column(tbl, lc, s[e][1], s[e][2], s[e][3], s[e][0], k[e][1]);
            const u32 n2 = column(tbl, lc, s[e][2], s[e][3], s[e][0], s[e][1], k[e][2]);
            const u32 n3 = column(tbl, lc, s[e][3], s[e][0], s[e][1], s[e][2], k[e][3]);
            s[e][0] = n0; s[e][1] = n1; s[e][2] = n2; s[e][3] = n3;
        }
#pragma unroll
        for (int e = 0; e < NS; ++e)
#pragma unroll
            for (int c = 0; c < 4; ++c) k[e][c] = nk[e][c];
    }
#pragma unroll
    for (int e = 0; e < NS; ++e) {
        out[e][0] = last_column(tbl, lc, s[e][0], s[e][1], s[e][2], s[e][3], k[e][0]);
        out[e][1] = last_column(tbl, lc, s[e][1], s[e][2], s[e][3], s[e][0], k[e][1]);
        out[e][2] = last_column(tbl, lc, s[e][2], s[e][3], s[e][0], s[e][1], k[e][2]);
        out[e][3] = last_column(tbl, lc, s[e][3], s[e][0], s[e][1], s[e][2], k[e][3]);
    }
}

struct T0Table {
    u32 v[256];
};

// floor(v / 2^d) of v read as a two's-complement integer
__device__ __forceinline__ u64 asr64(u64 v, int d) { return (u64)((int64_t)v >> d); }

// For the words j = first .. first + n - 1 of the PRF streams:
//   out = asr64((z ? z : 0) + (msg ? msg : 0) + [ALPHA] (F(self, j) - F(prev, j)), d)  -/+  [MASK] F(mask, j)
// (alpha under `nonce`, the mask stream under `mask_nonce`; the mask is subtracted unless add_mask), or, for
// binary shares (xor_mode, ALPHA only):  out = (z ? z : 0) ^ F(self, j) ^ F(prev, j).
// One thread handles one AES block = two consecutive words of each stream.
template <bool ALPHA, bool MASK>
__global__ __launch_bounds__(PRF_THREADS) void prf_combine_kernel(const u64* z, const u64* msg,
                                                          u64* out, size_t n, u64 first, u64 nonce,
                                                          u64 mask_nonce, int d, bool add_mask, bool xor_mode,
                                                          const PrfKeys keys, const T0Table table) {
    __shared__ __attribute__((aligned(16))) u32 tables[2 * 256 * 64];  // T0 then T2, one copy per bank
    {
        // thread t fills 16 of the 64 copies of entry t % 256 in both tables; consecutive threads
        // start at consecutive banks
        const int e = threadIdx.x & 255, q = threadIdx.x >> 8;
        const u32 v0 = table.v[e], v2 = (v0 << 16) | (v0 >> 16);
#pragma unroll 4
        for (int c = 0; c < 16; ++c) {
            const int copy = q * 16 + ((c + e) & 15);
            tables[e * 64 + copy] = v0;
            tables[256 * 64 + e * 64 + copy] = v2;
        }
    }
    __syncthreads();
    const char* tbl = reinterpret_cast<const char*>(tables);
    const u32 lc = ((threadIdx.x & 63) << 2) | 0x0100u;
    const u64 b_first = first >> 1, b_last = (first + n - 1) >> 1;  // n >= 1
    const u64 nblocks = b_last - b_first + 1;
    for (u64 bi = (u64)blockIdx.x * PRF_THREADS + threadIdx.x; bi < nblocks; bi += (u64)gridDim.x * PRF_THREADS) {
        const u64 block = b_first + bi;
        u64 w0 = 0, w1 = 0, r0 = 0, r1 = 0;
        constexpr int NS = (ALPHA ? 2 : 0) + (MASK ? 1 : 0);
        u32 in[NS][4], ct[NS][4];
        const u32* rk[NS];
        if constexpr (ALPHA) {
            rk[0] = keys.self;
            rk[1] = keys.prev;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                in[e][0] = (u32)block; in[e][1] = (u32)(block >> 32); in[e][2] = (u32)nonce; in[e][3] = (u32)(nonce >> 32);
            }
        }
        if constexpr (MASK) {
            rk[NS - 1] = keys.mask;
            in[NS - 1][0] = (u32)block; in[NS - 1][1] = (u32)(block >> 32);
            in[NS - 1][2] = (u32)mask_nonce; in[NS - 1][3] = (u32)(mask_nonce >> 32);
        }
        aes_blocks<NS>(tbl, lc, rk, in, ct);
        if constexpr (ALPHA) {
            const u64 a0 = ((u64)ct[0][1] << 32) | ct[0][0], a1 = ((u64)ct[0][3] << 32) | ct[0][2];
            const u64 b0 = ((u64)ct[1][1] << 32) | ct[1][0], b1 = ((u64)ct[1][3] << 32) | ct[1][2];
            w0 = xor_mode ? a0 ^ b0 : a0 - b0;
            w1 = xor_mode ? a1 ^ b1 : a1 - b1;
        }
        if constexpr (MASK) {
            r0 = ((u64)ct[NS - 1][1] << 32) | ct[NS - 1][0];
            r1 = ((u64)ct[NS - 1][3] << 32) | ct[NS - 1][2];
            if (!add_mask) { r0 = 0 - r0; r1 = 0 - r1; }
        }
        const u64 j0 = 2 * block, j1 = j0 + 1;  // word indices
        if (j0 >= first && j0 - first < n) {
            const size_t j = j0 - first;
            const u64 zj = z ? z[j] : 0;
            out[j] = xor_mode ? zj ^ w0 : asr64(zj + (msg ? msg[j] : 0) + w0, d) + r0;
        }
        if (j1 >= first && j1 - first < n) {
            const size_t j = j1 - first;
            const u64 zj = z ? z[j] : 0;
            out[j] = xor_mode ? zj ^ w1 : asr64(zj + (msg ? msg[j] : 0) + w1, d) + r1;
        }
    }
}

}  // namespace

hipError_t launch_prf_combine(const uint64_t* z, const uint64_t* msg, uint64_t* out, size_t n,
                              const uint8_t* key_self, const uint8_t* key_prev, uint64_t nonce, uint64_t first, int d,
                              const uint8_t* key_mask, uint64_t mask_nonce, bool add_mask, hipStream_t stream,
                              bool xor_mode) {
    if (n == 0) return hipSuccess;
    const bool alpha = key_self && key_prev, mask = key_mask != nullptr;
    if (!alpha && !mask) return hipErrorInvalidValue;
    if (xor_mode && (mask || msg || d != 0)) return hipErrorInvalidValue;
    PrfKeys keys = {};
    if (alpha) {
        expand_key(key_self, keys.self);
        expand_key(key_prev, keys.prev);
    }
    if (mask) expand_key(key_mask, keys.mask);
    T0Table table;
    memcpy(table.v, tables().t0, sizeof(table.v));
    // 128 KiB of tables per block: one block of 16 waves per compute unit, grid-stride beyond two rounds
    const size_t nblocks = (n + 1) / 2 + 1;
    size_t grid = (nblocks + PRF_THREADS - 1) / PRF_THREADS;
    if (grid > 256 * 2) grid = 256 * 2;
    const dim3 g((unsigned)grid), b(PRF_THREADS);
    if (alpha && mask)
        hipLaunchKernelGGL((prf_combine_kernel<true, true>), g, b, 0, stream, z, msg, out, n, (u64)first, (u64)nonce,
                           (u64)mask_nonce, d, add_mask, xor_mode, keys, table);
    else if (alpha)
        hipLaunchKernelGGL((prf_combine_kernel<true, false>), g, b, 0, stream, z, msg, out, n, (u64)first, (u64)nonce,
                           (u64)mask_nonce, d, add_mask, xor_mode, keys, table);
    else
        hipLaunchKernelGGL((prf_combine_kernel<false, true>), g, b, 0, stream, z, msg, out, n, (u64)first, (u64)nonce,
                           (u64)mask_nonce, d, add_mask, xor_mode, keys, table);
    return hipGetLastError();
}

hipError_t launch_zero_share(const uint64_t* z, uint64_t* out, size_t n, const uint8_t key_self[16],
                             const uint8_t key_prev[16], uint64_t nonce, uint64_t first, hipStream_t stream) {
    return launch_prf_combine(z, nullptr, out, n, key_self, key_prev, nonce, first, 0, nullptr, 0, false, stream, false);
}

}  // namespace cg
