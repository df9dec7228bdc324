// Philox4x32-10 (Salmon et al., SC'11) for the device.  One call yields the
// keys of four consecutive flat element indices.
#pragma once
#include "common.hpp"

namespace rad {

struct PhiloxKey { uint32_t k0, k1; };

__device__ __forceinline__ u32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    // three-input exclusive or in one instruction (v_bitop3_b32, truth table 0x96)
    const uint32_t n0 = __builtin_amdgcn_bitop3_b32((uint32_t)(p1 >> 32), c1, k0, 0x96);
    const uint32_t n2 = __builtin_amdgcn_bitop3_b32((uint32_t)(p0 >> 32), c3, k1, 0x96);
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  u32x4 out = {c0, c1, c2, c3};
  return out;
}

// keys of flat elements 4q .. 4q+3 of the tensor (stream_id, step)
__device__ __forceinline__ u32x4 element_quad_keys(uint64_t q, uint32_t stream_id, uint32_t step,
                                                   uint32_t seed_lo, uint32_t seed_hi) {
  return philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), stream_id, step, seed_lo, seed_hi);
}

}  // namespace rad
