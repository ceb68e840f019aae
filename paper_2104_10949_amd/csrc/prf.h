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

// out[j] = asr64((z ? z[j] : 0) + (msg ? msg[j] : 0) + alpha_j, d) -/+ F(key_mask, first + j), j < n, where
// alpha_j = F(key_self, first + j) - F(key_prev, first + j) under `nonce` if both keys are given (else 0), the
// mask stream runs under `mask_nonce` if key_mask is given (else no mask) and is subtracted unless add_mask;
// asr64 is the signed shift by d in [0, 63].  At least one of the two streams must be present.
// xor_mode (binary shares; alpha keys only, no msg, mask or shift): out[j] = (z ? z[j] : 0) ^ F(key_self, .) ^ F(key_prev, .).
hipError_t launch_prf_combine(const uint64_t* z, const uint64_t* msg, uint64_t* out, size_t n,
                              const uint8_t* key_self, const uint8_t* key_prev, uint64_t nonce, uint64_t first, int d,
                              const uint8_t* key_mask, uint64_t mask_nonce, bool add_mask, hipStream_t stream,
                              bool xor_mode = false);

}  // namespace cg
#endif
