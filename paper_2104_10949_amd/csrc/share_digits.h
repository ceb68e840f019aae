// Signed-digit split of 64-bit ring words and buffer views, shared by the product kernels.
#ifndef CG_SHARE_DIGITS_H
#define CG_SHARE_DIGITS_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cg {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));
typedef unsigned int u2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32;
typedef uint64_t u64;

// voffset that is out of range for every buffer view (views are < 2^31 bytes):
// the hardware then returns zeros instead of reading memory.
static constexpr u32 OOB = 0x80000000u;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, u32 bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
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

}  // namespace cg
#endif
