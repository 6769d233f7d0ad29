// Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
// as 1, 2, 3", SC'11, Sec. 3.3): ten rounds of two 32x32->64 multiplies and a
// word permutation, keys advanced by Weyl constants between rounds.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace nat {

struct u32x4 { uint32_t x, y, z, w; };

__device__ __forceinline__ u32x4 philox4x32_10(u32x4 ctr, uint32_t k0, uint32_t k1) {
  constexpr uint32_t kMulA = 0xD2511F53u, kMulB = 0xCD9E8D57u;
  constexpr uint32_t kWeylA = 0x9E3779B9u, kWeylB = 0xBB67AE85u;
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint32_t hiA = __umulhi(kMulA, ctr.x), loA = kMulA * ctr.x;
    const uint32_t hiB = __umulhi(kMulB, ctr.z), loB = kMulB * ctr.z;
    ctr = u32x4{hiB ^ ctr.y ^ k0, loB, hiA ^ ctr.w ^ k1, loA};
    k0 += kWeylA;
    k1 += kWeylB;
  }
  return ctr;
}

}  // namespace nat
