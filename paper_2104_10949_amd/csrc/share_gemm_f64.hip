// Comparator for the limb choice: the party's three-term product computed the way
// Sec. II-B embeds ring arithmetic in floating point, on the float64 matrix instruction.
//
// A 64-bit word is cut into k = 4 unsigned blocks of w = 16 bits, each held as a
// double; a*b mod 2^64 = sum over block pairs (i, j) with 16(i + j) < 64, i.e. i + j <= 3
// (10 pairs), of a_i b_j 2^(16(i+j)).  Every block product is below 2^32, so a float64
// accumulator stays exact while it has received fewer than 2^20 of them (the paper's
// bound, from 52 bits of precision); pairs of equal i + j share an accumulator, which
// then receives (i + j + 1) products per contraction index and operand pair.  The
// accumulators are folded into the 64-bit result every SEG contraction indices.
//
// As in the int8 kernel the three terms are two ring products,
// x_a (w_a + w_b) + x_b w_a, so one (m, n, k) costs 20 float64 MACs on
// v_mfma_f64_16x16x4_f64.  The kernel is a plain tiled product: it exists to put a
// measured number next to the int8 route, not to be tuned beyond being matrix-core bound.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "share_gemm.h"

namespace cg {

namespace {

typedef uint64_t u64;
typedef double v4d __attribute__((ext_vector_type(4)));

constexpr int F_BM = 64, F_BN = 64;  // block tile: 4 waves as 2 x 2, each wave 32 x 32 = 2 x 2 instruction tiles
constexpr int F_KS = 8;              // contraction indices per staged chunk
constexpr int F_NT = 256;
// (3 + 1) pairs * 2 operand pairs * SEG products of < 2^32 each stay below 2^52
constexpr int F_SEG = 1 << 15;

// LDS: [operand][block of 16 bits][k][row] doubles; operands: x_a, x_b, w_a + w_b, w_a
constexpr int F_PLANE = F_KS * F_BM;  // doubles of one block plane (F_BM == F_BN)

__device__ __forceinline__ void split_store(double* dst, u64 v) {
#pragma unroll
    for (int b = 0; b < 4; ++b) dst[b * F_PLANE] = (double)(uint32_t)((v >> (16 * b)) & 0xFFFFu);
}

__global__ __launch_bounds__(F_NT) void share_gemm_f64limb_kernel(const u64* __restrict__ x_a,
                                                                  const u64* __restrict__ x_b,
                                                                  const u64* __restrict__ w_a,
                                                                  const u64* __restrict__ w_b, u64* __restrict__ z,
                                                                  int M, int N, int K) {
    __shared__ double lds[4 * 4 * F_PLANE];  // 64 KB
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int tiles_n = (N + F_BN - 1) / F_BN;
    const int m0 = (int)(blockIdx.x / tiles_n) * F_BM, n0 = (int)(blockIdx.x % tiles_n) * F_BN;

    // staging: thread t fetches contraction indices t / 64 and t / 64 + 4 of row t % 64 of every operand, so that a
    // wave's LDS stores of one block plane are consecutive doubles
    const int kq = tid >> 6, r0 = tid & 63;
    u64 sx_a[2], sx_b[2], sw_s[2], sw_a[2];
    auto fetch = [&](int kc) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int k = kc + kq + 4 * h;
            const int row = m0 + r0, col = n0 + r0;
            const bool va = row < M && k < K, vb = col < N && k < K;
            const size_t ia = (size_t)row * (size_t)K + (size_t)k, ib = (size_t)col * (size_t)K + (size_t)k;
            sx_a[h] = va ? x_a[ia] : 0;
            sx_b[h] = va ? x_b[ia] : 0;
            const u64 wa = vb ? w_a[ib] : 0, wb = vb ? w_b[ib] : 0;
            sw_s[h] = wa + wb;
            sw_a[h] = wa;
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int o = (kq + 4 * h) * F_BM + r0;
            split_store(lds + 0 * 4 * F_PLANE + o, sx_a[h]);
            split_store(lds + 1 * 4 * F_PLANE + o, sx_b[h]);
            split_store(lds + 2 * 4 * F_PLANE + o, sw_s[h]);
            split_store(lds + 3 * 4 * F_PLANE + o, sw_a[h]);
        }
    };

    // instruction operands: lane l supplies A[row l % 16][k l / 16] and B[k l / 16][col l % 16];
    // accumulator register i of lane l is C[row 4 i + l / 16][col l % 16]
    const int fr = lane & 15, fk = lane >> 4;
    v4d acc[4][2][2];
    auto clear = [&]() {
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b) acc[s][a][b] = v4d{0.0, 0.0, 0.0, 0.0};
    };
    auto fold = [&](bool accumulate) {
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int row = m0 + wm * 32 + a * 16 + 4 * i + fk, col = n0 + wn * 32 + b * 16 + fr;
                    u64 v = 0;
#pragma unroll
                    for (int s = 0; s < 4; ++s) v += (u64)acc[s][a][b][i] << (16 * s);
                    if (row < M && col < N) {
                        u64* dst = z + (size_t)row * (size_t)N + (size_t)col;
                        if (accumulate) v += *dst;
                        *dst = v;
                    }
                }
    };

    clear();
    fetch(0);
    int seg_begin = 0;
    for (int kc = 0; kc < K; kc += F_KS) {
        __syncthreads();  // the previous chunk's reads are done
        stage();
        __syncthreads();
        if (kc + F_KS < K) fetch(kc + F_KS);
#pragma unroll
        for (int kk = 0; kk < F_KS; kk += 4) {
#pragma unroll
            for (int half = 0; half < 2; ++half) {  // x_a against w_a + w_b, then x_b against w_a
                const double* pa = lds + (half ? 1 : 0) * 4 * F_PLANE + (kk + fk) * F_BM + wm * 32 + fr;
                const double* pb = lds + (half ? 3 : 2) * 4 * F_PLANE + (kk + fk) * F_BN + wn * 32 + fr;
                double fa[4][2], fb[4][2];
#pragma unroll
                for (int blk = 0; blk < 4; ++blk)
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        fa[blk][t] = pa[blk * F_PLANE + 16 * t];
                        fb[blk][t] = pb[blk * F_PLANE + 16 * t];
                    }
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; i + j < 4; ++j)
#pragma unroll
                        for (int a = 0; a < 2; ++a)
#pragma unroll
                            for (int b = 0; b < 2; ++b)
                                acc[i + j][a][b] = __builtin_amdgcn_mfma_f64_16x16x4f64(fa[i][a], fb[j][b],
                                                                                        acc[i + j][a][b], 0, 0, 0);
            }
        }
        if (kc + F_KS - seg_begin >= F_SEG && kc + F_KS < K) {
            fold(seg_begin > 0);
            clear();
            seg_begin = kc + F_KS;
        }
    }
    fold(seg_begin > 0);
}

}  // namespace

hipError_t launch_share_gemm_f64limb(const uint64_t* x_a, const uint64_t* x_b, const uint64_t* w_a,
                                     const uint64_t* w_b, uint64_t* z, int M, int N, int K, hipStream_t stream) {
    const int64_t tiles = (int64_t)((M + F_BM - 1) / F_BM) * (int64_t)((N + F_BN - 1) / F_BN);
    if (tiles > 0x7FFFFFFF) return hipErrorInvalidValue;
    hipLaunchKernelGGL(share_gemm_f64limb_kernel, dim3((unsigned)tiles), dim3(F_NT), 0, stream, x_a, x_b, w_a, w_b, z, M,
                       N, K);
    return hipGetLastError();
}

}  // namespace cg
