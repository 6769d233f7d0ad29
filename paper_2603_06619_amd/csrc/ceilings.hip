// Measurement aids: the two practical ceilings the loss stage is priced against, as kernels of
// known work so that a benchmark or a counter run can time them beside the library's own kernels.
//   nat_probe_mfma_bf16  matrix-core throughput with operands held in registers (no memory traffic
//                        in the loop): constant operands reach the nominal clock, pseudo-random
//                        operand bits show the rate the power limit allows on real data;
//   nat_probe_copy       a plain 16-byte-per-lane copy: HBM bandwidth, and the known-size kernel
//                        against which byte counters are scaled.
// Neither is on the product path.
#include "nat_internal.h"

namespace nat {

typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));
typedef short probe_s16x8 __attribute__((ext_vector_type(8)));
typedef float probe_f32x16 __attribute__((ext_vector_type(16)));

constexpr int kProbeBlocks = 256 * 8;             // eight workgroups per compute unit in sequence
constexpr int kProbeThreads = 256;                // one wavefront per SIMD, 256 accumulator registers each

// 16 independent 32x32x16 products per iteration and wavefront: the accumulator tile of the GEMM core.
__global__ void __launch_bounds__(kProbeThreads, 1)
probe_mfma_kernel(float* __restrict__ out, int iters, int random_operands) {
  probe_f32x16 acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  probe_bf16x8 a[4], b[4];
  unsigned x = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 17u;
#pragma unroll
  for (int f = 0; f < 4; ++f) {
    probe_s16x8 ra, rb;
#pragma unroll
    for (int i = 0; i < 8; ++i) {                 // values in +-[1, 2): sign and mantissa bits random
      x = x * 1664525u + 1013904223u;
      ra[i] = random_operands ? (short)(((x >> 16) & 0x807f) | 0x3f80) : (short)0x3f80;
      x = x * 1664525u + 1013904223u;
      rb[i] = random_operands ? (short)(((x >> 16) & 0x807f) | 0x3f80) : (short)0x3f80;
    }
    a[f] = __builtin_bit_cast(probe_bf16x8, ra);
    b[f] = __builtin_bit_cast(probe_bf16x8, rb);
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i * 4 + j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i * 4 + j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  out[(size_t)blockIdx.x * kProbeThreads + threadIdx.x] = s;
}

__global__ void __launch_bounds__(256)
probe_copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace nat

using namespace nat;

extern "C" size_t nat_probe_mfma_scratch_bytes(void) { return (size_t)kProbeBlocks * kProbeThreads * sizeof(float); }

extern "C" nat_status nat_probe_mfma_bf16(int32_t random_operands, int32_t iters, float* d_scratch,
                                          double* h_flops, void* stream) {
  if (!d_scratch || iters <= 0) return NAT_INVALID_ARG;
  probe_mfma_kernel<<<kProbeBlocks, kProbeThreads, 0, (hipStream_t)stream>>>(d_scratch, iters, random_operands);
  NAT_LAUNCH_CHECK();
  // blocks x 4 wavefronts x iterations x 16 products of 2 * 32 * 32 * 16 flops
  if (h_flops) *h_flops = (double)kProbeBlocks * 4.0 * (double)iters * 16.0 * 32768.0;
  return NAT_OK;
}

extern "C" nat_status nat_probe_copy(void* d_dst, const void* d_src, size_t bytes, void* stream) {
  if (!d_dst || !d_src || (bytes & 15) || ((uintptr_t)d_dst & 15) || ((uintptr_t)d_src & 15)) return NAT_INVALID_ARG;
  if (bytes == 0) return NAT_OK;
  const size_t n16 = bytes / 16;
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 256 * 32) blocks = 256 * 32;
  probe_copy_kernel<<<(unsigned)blocks, 256, 0, (hipStream_t)stream>>>((uint4*)d_dst, (const uint4*)d_src, n16);
  NAT_LAUNCH_CHECK();
  return NAT_OK;
}
