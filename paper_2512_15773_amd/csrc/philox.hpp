// Philox4x32-10 (Salmon et al., SC'11) and the noise streams of the speculative round.
// counter = (block, timestep, environment id, stream); key = 64-bit seed.
// stream 0: Gaussian noise xi (block i -> elements 4i..4i+3), stream 1: acceptance uniform (word 0).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tsdp {

struct u32x4 { uint32_t x, y, z, w; };

__device__ __forceinline__ u32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  return {c0, c1, c2, c3};
}

// top 23 bits + 1/2, scaled by 2^-23: strictly inside (0,1) and exact in fp32
__device__ __forceinline__ float u01(uint32_t w) { return ((float)(w >> 9) + 0.5f) * 1.1920928955078125e-07f; }

// four standard normals of block `blk` of xi_{env,t} (Box-Muller on word pairs)
__device__ __forceinline__ float4 xi_block(uint64_t seed, int env, int t, int blk) {
  const u32x4 w = philox4x32_10((uint32_t)blk, (uint32_t)t, (uint32_t)env, 0u, (uint32_t)seed, (uint32_t)(seed >> 32));
  const float r0 = sqrtf(-2.0f * logf(u01(w.x)));
  const float r1 = sqrtf(-2.0f * logf(u01(w.z)));
  float s0, c0, s1, c1;
  sincospif(2.0f * u01(w.y), &s0, &c0);
  sincospif(2.0f * u01(w.w), &s1, &c1);
  return make_float4(r0 * c0, r0 * s0, r1 * c1, r1 * s1);
}

__device__ __forceinline__ float accept_uniform(uint64_t seed, int env, int t) {
  const u32x4 w = philox4x32_10(0u, (uint32_t)t, (uint32_t)env, 1u, (uint32_t)seed, (uint32_t)(seed >> 32));
  return u01(w.x);
}

}  // namespace tsdp
