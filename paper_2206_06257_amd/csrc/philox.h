// Philox4x32-10 counter-based generator (Salmon et al., SC'11) for the device side:
// ten rounds of two 32x32 -> 64-bit multiplies; the key walks a Weyl sequence.
// One call yields the four 32-bit words of block `blk` of stream `stream_id` under `seed`.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dat {

struct PhiloxWords { uint32_t w0, w1, w2, w3; };

__device__ __forceinline__ PhiloxWords philox_block(uint64_t blk, uint64_t seed, uint32_t stream_id) {
  uint32_t c0 = (uint32_t)blk, c1 = (uint32_t)(blk >> 32), c2 = stream_id, c3 = 0u;
  uint32_t ka = (uint32_t)seed, kb = (uint32_t)(seed >> 32);
#pragma unroll
  for (int i = 0; i < 10; ++i) {
    // one 32x32 -> 64-bit multiply per product (a single v_mad_u64_u32 instead of a hi/lo pair)
    const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
    const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    c0 = hi1 ^ c1 ^ ka;
    c1 = lo1;
    c2 = hi0 ^ c3 ^ kb;
    c3 = lo0;
    ka += 0x9E3779B9u;
    kb += 0xBB67AE85u;
  }
  return PhiloxWords{c0, c1, c2, c3};
}

// 24-bit uniform in [0,1): top 24 bits of a word times 2^-24 (exact in fp32).
__device__ __forceinline__ float u24(uint32_t w) { return (float)(w >> 8) * 5.9604644775390625e-8f; }

}  // namespace dat
