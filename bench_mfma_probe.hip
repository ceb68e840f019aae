// Register-only int8 MFMA issue loop: the matrix-core rate this chip sustains for
// given operand bytes, with no memory traffic in the loop.  Used by bench.py to
// report the share-product kernel against a MEASURED ceiling next to the
// published one: operand bit patterns change the power drawn and with it the
// clock, and secret shares are uniformly random bytes.  Built next to bench.py; not part of libcg.so.
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Eight rotating accumulators, as in the share-product kernel; operands are read
// once from `src` (16 bytes per lane and operand) before the loop.
template <int NT>
__global__ __launch_bounds__(NT) void mfma_rate_kernel(const v4i* __restrict__ src, int* __restrict__ sink,
                                                       int iters) {
    const int t = threadIdx.x;
    v4i a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = src[(t * 8 + i) & 4095];
        b[i] = src[(t * 8 + 4 + i) & 4095];
    }
    v16i c[8];
#pragma unroll
    for (int s = 0; s < 8; ++s)
#pragma unroll
        for (int i = 0; i < 16; ++i) c[s][i] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < 8; ++s)
            c[s] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[s & 3], b[(s >> 1) & 3], c[s], 0, 0, 0);
    }
    int acc = 0;
#pragma unroll
    for (int s = 0; s < 8; ++s)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc += c[s][i];
    sink[(size_t)blockIdx.x * NT + t] = acc;
}

// The same loop on v_mfma_i32_16x16x64_i8, the instruction the share-product kernel issues: 32 rotating
// accumulators of four registers (as many accumulator registers as above), half the MACs per instruction.
template <int NT>
__global__ __launch_bounds__(NT) void mfma16_rate_kernel(const v4i* __restrict__ src, int* __restrict__ sink,
                                                         int iters) {
    const int t = threadIdx.x;
    v4i a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = src[(t * 8 + i) & 4095];
        b[i] = src[(t * 8 + 4 + i) & 4095];
    }
    v4i c[32];
#pragma unroll
    for (int s = 0; s < 32; ++s) c[s] = v4i{0, 0, 0, 0};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < 32; ++s)
            c[s] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[s & 3], b[(s >> 1) & 3], c[s], 0, 0, 0);
    }
    int acc = 0;
#pragma unroll
    for (int s = 0; s < 32; ++s) acc += c[s][0] + c[s][1] + c[s][2] + c[s][3];
    sink[(size_t)blockIdx.x * NT + t] = acc;
}

// The same loop for the float64 matrix instruction the paper's 16-bit-limb embedding
// would run on (v_mfma_f64_16x16x4_f64: 16*16*4 MACs per instruction and wave).
typedef double v4d __attribute__((ext_vector_type(4)));

template <int NT>
__global__ __launch_bounds__(NT) void mfma_f64_rate_kernel(const double* __restrict__ src, double* __restrict__ sink,
                                                           int iters) {
    const int t = threadIdx.x;
    double a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = src[(t * 8 + i) & 8191];
        b[i] = src[(t * 8 + 4 + i) & 8191];
    }
    v4d c[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) c[s] = v4d{0.0, 0.0, 0.0, 0.0};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < 8; ++s)
            c[s] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[s & 3], b[(s >> 1) & 3], c[s], 0, 0, 0);
    }
    double acc = 0.0;
#pragma unroll
    for (int s = 0; s < 8; ++s) acc += c[s][0] + c[s][1] + c[s][2] + c[s][3];
    sink[(size_t)blockIdx.x * NT + t] = acc;
}

extern "C" {

// Launch the loop on `blocks` blocks of 4*waves_per_simd waves.
//   operands : device, 64 KiB of operand bytes (4096 x 16 B)
//   sink     : device, blocks * 256 * waves_per_simd ints, receives a checksum
// Each wave issues 8*iters MFMAs of 32*32*32 MACs.  Returns 0 on success, 1 on bad
// arguments, 2 if the launch failed.  The caller times the stream.
__attribute__((visibility("default")))
int cg_probe_mfma_rate(const void* operands, void* sink, int blocks, int waves_per_simd, int iters,
                       void* stream) {
    if (!operands || !sink || blocks < 1 || iters < 1 || (waves_per_simd != 1 && waves_per_simd != 2)) return 1;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (waves_per_simd == 1)
        hipLaunchKernelGGL(mfma_rate_kernel<256>, dim3(blocks), dim3(256), 0, s,
                           static_cast<const v4i*>(operands), static_cast<int*>(sink), iters);
    else
        hipLaunchKernelGGL(mfma_rate_kernel<512>, dim3(blocks), dim3(512), 0, s,
                           static_cast<const v4i*>(operands), static_cast<int*>(sink), iters);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

// The 16x16x64 form: each wave issues 32*iters MFMAs of 16*16*64 MACs; arguments as cg_probe_mfma_rate.
__attribute__((visibility("default")))
int cg_probe_mfma16_rate(const void* operands, void* sink, int blocks, int waves_per_simd, int iters,
                         void* stream) {
    if (!operands || !sink || blocks < 1 || iters < 1 || (waves_per_simd != 1 && waves_per_simd != 2)) return 1;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (waves_per_simd == 1)
        hipLaunchKernelGGL(mfma16_rate_kernel<256>, dim3(blocks), dim3(256), 0, s,
                           static_cast<const v4i*>(operands), static_cast<int*>(sink), iters);
    else
        hipLaunchKernelGGL(mfma16_rate_kernel<512>, dim3(blocks), dim3(512), 0, s,
                           static_cast<const v4i*>(operands), static_cast<int*>(sink), iters);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

// float64 variant: `operands` holds 8192 doubles (16-bit integers as doubles keep the
// sums exact, as in the paper's embedding), `sink` blocks * 256 * waves_per_simd doubles.
// Each wave issues 8*iters MFMAs of 16*16*4 MACs.
__attribute__((visibility("default")))
int cg_probe_mfma_f64_rate(const void* operands, void* sink, int blocks, int waves_per_simd, int iters,
                           void* stream) {
    if (!operands || !sink || blocks < 1 || iters < 1 || (waves_per_simd != 1 && waves_per_simd != 2)) return 1;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (waves_per_simd == 1)
        hipLaunchKernelGGL(mfma_f64_rate_kernel<256>, dim3(blocks), dim3(256), 0, s,
                           static_cast<const double*>(operands), static_cast<double*>(sink), iters);
    else
        hipLaunchKernelGGL(mfma_f64_rate_kernel<512>, dim3(blocks), dim3(512), 0, s,
                           static_cast<const double*>(operands), static_cast<double*>(sink), iters);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

}  // extern "C"
