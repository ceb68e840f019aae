// The party's local product (CryptGPU Sec. III-B, "Multiplication" and "Convolutions and matrix
// multiplication") for a left operand of few rows: fully connected layers at small batch.
//
// Such a product is a few microseconds of matrix work, so what counts is the length of the chain
// launch -> load -> split -> multiply -> store and how many compute units share it, not the rate of any
// unit.  A block owns one 16 x 16 block of z; its waves share out the 32-word slices of K and never wait for
// each other until the end.  For v_mfma_i32_16x16x64_i8 a lane supplies 16 contraction bytes of one row, so
// lane (r, g) ends up with the sixteen words of row r that make up k-group g (g = 2 * share + half of the
// slice), splits them into eight signed digits in its own registers (which is the operand layout of the
// instruction), and the wave issues the 36 digit-pair products of the slice.  The waves' partial results
// meet in a 2 KB LDS tile through 64-bit LDS adds; one plain store per element, or an atomic add when K is
// also split over blocks.
// Same arithmetic as share_gemm_kernel: digits, accumulators P_0..P_7, one fold at the end (the launcher takes
// products of at most 511 slices per wave).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "share_digits.h"
#include "share_gemm.h"

namespace cg {
namespace {

constexpr int SMALL_WAVES = 8;        // waves of a block: two per SIMD, 256 registers each
constexpr int SMALL_MAX_SLICES = 511 * SMALL_WAVES;  // a wave's i32 accumulators stay exact for 511 slices (see share_gemm.hip)
// Which products the launcher takes (measured against share_gemm_kernel at M = 8, 32, 64, N = 64 .. 4096,
// K = 128 .. 25088): with one 16-row block every shape up to the slice limit (4.4 us against 13 us at K = 128,
// 281 against 379 us at 8 x 4096 x 25088); with two to four row blocks the right operand is read once per row
// block, and the tiled kernel wins from about 4600 (16 x 16 block, slice) units on.
constexpr int SMALL_MAX_ROWS = 64;
constexpr int SMALL_ONE_BLOCK_ROWS = 16;
constexpr int64_t SMALL_MAX_UNITS = 4608;
// K is split over blocks as well until the grid has this many blocks (one block per compute unit fits)
constexpr int64_t SMALL_TARGET_BLOCKS = 256;

// Sixteen words (eight 16-byte registers, word 2i in v[i].xy and word 2i+1 in v[i].zw) -> eight digit
// registers: byte 4j + t of d[l] is digit l of word 4j + t.
__device__ __forceinline__ void split16(u4 (&v)[8], v4i (&d)[8]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        u32 lo[4] = {v[2 * j].x, v[2 * j].z, v[2 * j + 1].x, v[2 * j + 1].z};
        u32 hi[4] = {v[2 * j].y, v[2 * j].w, v[2 * j + 1].y, v[2 * j + 1].w};
#pragma unroll
        for (int t = 0; t < 4; ++t) recode(lo[t], hi[t]);
        u32 dl[4], dh[4];
        transpose4(lo[0], lo[1], lo[2], lo[3], dl);
        transpose4(hi[0], hi[1], hi[2], hi[3], dh);
#pragma unroll
        for (int l = 0; l < 4; ++l) {
            d[l][j] = (int)dl[l];
            d[4 + l][j] = (int)dh[l];
        }
    }
}

__device__ __forceinline__ u4 add64x2(u4 a, u4 b) {
    const u64 s0 = (((u64)a.y << 32) | a.x) + (((u64)b.y << 32) | b.x);
    const u64 s1 = (((u64)a.w << 32) | a.z) + (((u64)b.w << 32) | b.z);
    u4 r;
    r.x = (u32)s0; r.y = (u32)(s0 >> 32); r.z = (u32)s1; r.w = (u32)(s1 >> 32);
    return r;
}

// grid: x = 16-column block of z, y = 16-row block, z = range of K slices (gridDim.z > 1: z is cleared or
// holds the value to add to, and every block adds atomically).  Rows of the operands past M or N are
// replaced by the last row: their products land in elements that are never stored.
//
// A slice on its way to the matrix instruction.  Memory wants neighbouring lanes on neighbouring bytes, the
// instruction wants lane (r, g) to hold words of row r only, so the raw words cross a wave-private LDS
// buffer: four regions (x_a, x_b, w_a + w_b, w_a) of 16 rows x 256 bytes.  Loads and LDS writes run with sixteen
// lanes along the sixteen 16-byte pieces of a row's slice (four rows per instruction); the read-back has lane
// (r, g) take the eight pieces of half g & 1 of row r in region g >> 1.  Piece p of row r sits at piece p ^ r, so
// that neither the sixteen pieces of a row nor one piece of sixteen rows fall on the same banks.  No barrier is
// involved: a wave reads what it wrote itself.
__global__ __launch_bounds__(SMALL_WAVES * 64) void share_gemm_small_kernel(const GemmParams p) {
    __shared__ __attribute__((aligned(16))) char stage[SMALL_WAVES][4][16 * 256];
    __shared__ unsigned long long red[256];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // said to be uniform: the slice loop runs on the scalar unit
    if (tid < 256) red[tid] = 0;
    __syncthreads();

    const int n0 = blockIdx.x * 16, m0 = blockIdx.y * 16;
    const u32 K = (u32)p.K;
    const int nk = (int)((K + 31) >> 5);
    const int per = (nk + (int)gridDim.z - 1) / (int)gridDim.z;
    const int ks_begin = (int)blockIdx.z * per;
    const int ks_end = ks_begin + per < nk ? ks_begin + per : nk;

    // loading side: piece lp of rows lr, lr + 4, lr + 8, lr + 12 of the block, through buffer views (the whole left
    // operand; the right operand from the block's first row on) whose range check turns an offset of OOB into zeros
    const int lp = lane & 15, lr = lane >> 4;
    const u64 b_left = (u64)(p.N - n0) * K * 8u;
    const __amdgpu_buffer_rsrc_t rs_xa = make_rsrc(p.x_a, (u32)((u64)p.M * K * 8u)),
                                 rs_xb = make_rsrc(p.x_b, (u32)((u64)p.M * K * 8u)),
                                 rs_wa = make_rsrc(p.w_a + (u64)n0 * K, b_left > 0x7FFFFFFFull ? 0x7FFFFFFFu : (u32)b_left),
                                 rs_wb = make_rsrc(p.w_b + (u64)n0 * K, b_left > 0x7FFFFFFFull ? 0x7FFFFFFFu : (u32)b_left);
    u32 a_off[4], b_off[4];
    int st_off[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int r = 4 * j + lr;
        a_off[j] = (u32)(m0 + r < p.M ? m0 + r : p.M - 1) * K * 8u + 16u * lp;
        b_off[j] = (u32)(n0 + r < p.N ? r : p.N - 1 - n0) * K * 8u + 16u * lp;
        st_off[j] = r * 256 + ((lp ^ r) << 4);
    }
    // multiplying side: lane (r16, kg)
    const int r16 = lane & 15, kg = lane >> 4;
    char* const my_stage = &stage[wave][0][0];
    const char* const rd = my_stage + (kg >> 1) * 4096 + r16 * 256;   // x_a / x_b, and + 8192: w_a + w_b / w_a
    int rd_off[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) rd_off[i] = ((8 * (kg & 1) + i) ^ r16) << 4;

    u4 rxa[4], rxb[4], rwa[4], rwb[4];
    // words 2 lp, 2 lp + 1 of slice ks of the four rows (K is even: the pair is inside or outside K as a whole)
    auto load = [&](int ks) {
        const u32 at = (32u * (u32)ks + 2u * (u32)lp < K ? 0u : OOB) + 256u * (u32)ks;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            rxa[j] = __builtin_amdgcn_raw_buffer_load_b128(rs_xa, a_off[j] + at, 0, 0);
            rxb[j] = __builtin_amdgcn_raw_buffer_load_b128(rs_xb, a_off[j] + at, 0, 0);
            rwa[j] = __builtin_amdgcn_raw_buffer_load_b128(rs_wa, b_off[j] + at, 0, 0);
            rwb[j] = __builtin_amdgcn_raw_buffer_load_b128(rs_wb, b_off[j] + at, 0, 0);
        }
    };

    v4i acc[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) acc[s] = v4i{0, 0, 0, 0};
    int ks = ks_begin + wave;
    if (ks < ks_end) load(ks);
    while (ks < ks_end) {   // uniform over the wave
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            *reinterpret_cast<u4*>(my_stage + st_off[j]) = rxa[j];
            *reinterpret_cast<u4*>(my_stage + 4096 + st_off[j]) = rxb[j];
            *reinterpret_cast<u4*>(my_stage + 8192 + st_off[j]) = add64x2(rwa[j], rwb[j]);
            *reinterpret_cast<u4*>(my_stage + 12288 + st_off[j]) = rwa[j];
        }
        const int next = ks + SMALL_WAVES;
        if (next < ks_end) load(next);
        __builtin_amdgcn_wave_barrier();   // (compiler only) the reads below follow the writes above
        u4 ra[8], rb[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            ra[i] = *reinterpret_cast<const u4*>(rd + rd_off[i]);
            rb[i] = *reinterpret_cast<const u4*>(rd + 8192 + rd_off[i]);
        }
        __builtin_amdgcn_wave_barrier();
        v4i ad[8], bd[8];
        split16(ra, ad);
        split16(rb, bd);
#pragma unroll
        for (int l = 0; l < 8; ++l)
#pragma unroll
            for (int m = 0; m + l < 8; ++m)
                acc[l + m] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ad[l], bd[m], acc[l + m], 0, 0, 0);
        ks = next;
    }
    // fold: sum_s sext(P_s) << 8s, P_4..P_7 only reach bits 32..63; lane (c, g) holds rows 4g .. 4g+3 of
    // column c of the block
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        u64 v = (u64)(int64_t)acc[0][i];
        v += (u64)(int64_t)acc[1][i] << 8;
        v += (u64)(int64_t)acc[2][i] << 16;
        v += (u64)(int64_t)acc[3][i] << 24;
        const u32 hi = (u32)acc[4][i] + ((u32)acc[5][i] << 8) + ((u32)acc[6][i] << 16) + ((u32)acc[7][i] << 24);
        v += (u64)hi << 32;
        atomicAdd(&red[(4 * kg + i) * 16 + r16], (unsigned long long)v);
    }
    __syncthreads();
    if (tid < 256) {
        const int row = m0 + (tid >> 4), col = n0 + (tid & 15);
        if (row < p.M && col < p.N) {
            u64* dst = p.z + (u64)row * (u64)p.N + (u64)col;
            const u64 v = red[tid];
            if (gridDim.z > 1) atomicAdd(reinterpret_cast<unsigned long long*>(dst), (unsigned long long)v);
            else *dst = p.z_add ? *dst + v : v;
        }
    }
}

}  // namespace

// Row-major operands with 16-byte loads (K even, 16-byte aligned bases), few rows on the left, and a K whose
// slices, shared out over a block's waves, fit one fold.
bool share_gemm_small_applies(const GemmParams& p) {
    const int64_t nk = (p.K + 31) / 32;
    if (p.lda != p.K || nk > SMALL_MAX_SLICES || p.M > SMALL_MAX_ROWS) return false;
    if ((p.N + 15) / 16 > (1 << 20)) return false;   // grid size in threads stays below 2^32
    if (p.M <= SMALL_ONE_BLOCK_ROWS) return true;
    return (int64_t)((p.M + 15) / 16) * ((p.N + 15) / 16) * nk <= SMALL_MAX_UNITS;
}

hipError_t launch_share_gemm_small(const GemmParams& p, hipStream_t stream) {
    const int64_t tiles_m = (p.M + 15) / 16, tiles_n = (p.N + 15) / 16, tiles = tiles_m * tiles_n;
    const int nk = (p.K + 31) / 32;
    // K is split over blocks as well when the blocks of z alone would leave compute units idle, as long as a
    // wave keeps at least two slices
    int64_t ksplit = 1;
    if (tiles < SMALL_TARGET_BLOCKS) {
        ksplit = (SMALL_TARGET_BLOCKS + tiles - 1) / tiles;
        const int64_t most = nk / (2 * SMALL_WAVES);
        if (ksplit > most) ksplit = most;
        if (ksplit < 1) ksplit = 1;
    }
    if (ksplit > 1 && !p.z_prezeroed && !p.z_add)
        if (hipError_t e = launch_zero_words(p.z, (size_t)p.M * (size_t)p.N, stream)) return e;
    hipLaunchKernelGGL(share_gemm_small_kernel, dim3((unsigned)tiles_n, (unsigned)tiles_m, (unsigned)ksplit),
                       dim3(SMALL_WAVES * 64), 0, stream, p);
    return hipGetLastError();
}

}  // namespace cg
