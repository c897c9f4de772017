// Philox4x32-10 on the device, from its published definition (Salmon, Moraes,
// Dror, Shaw, SC'11, Section 3.3): counter (c0..c3), key (k0,k1), ten rounds of
// {two 32x32->64 multiplies, cross XOR with the odd counter words and the key,
// word permutation}, key advanced by two Weyl constants between rounds.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pbt {

enum {
  DOMAIN_BATCH = 1,
  DOMAIN_DONOR = 2,
  DOMAIN_EXPLORE = 3,
  DOMAIN_INIT_W = 4,
  DOMAIN_INIT_H = 5,
  DOMAIN_LATENT = 6,
  DOMAIN_DROPOUT = 16,
};

struct u32x4 { uint32_t x, y, z, w; };

__host__ __device__ inline u32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                               uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return u32x4{c0, c1, c2, c3};
}

// floor(x * n / 2^32): an index in [0, n).
__host__ __device__ inline uint32_t philox_bounded(uint32_t x, uint32_t n) {
  return (uint32_t)(((uint64_t)x * (uint64_t)n) >> 32);
}

// (x + 0.5) / 2^32: a double in the open interval (0, 1).
__host__ __device__ inline double philox_unit(uint32_t x) { return ((double)x + 0.5) * (1.0 / 4294967296.0); }

}  // namespace pbt
