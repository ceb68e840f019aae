// Internal interface of the PRF / reshare kernels.
#ifndef CG_PRF_H
#define CG_PRF_H

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace cg {

// out[j] = (z ? z[j] : 0) + F(key_self, first + j) - F(key_prev, first + j), j < n.
// z and out are device pointers (may be equal); keys are host pointers.
hipError_t launch_zero_share(const uint64_t* z, uint64_t* out, size_t n, const uint8_t key_self[16],
                             const uint8_t key_prev[16], uint64_t nonce, uint64_t first, hipStream_t stream);

}  // namespace cg
#endif
