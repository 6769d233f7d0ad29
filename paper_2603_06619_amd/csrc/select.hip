// nat_advantage and nat_select: group-relative advantage (Eq. 2) and the token
// selection mask of Sec. 3.1 (URS) and Sec. 4 (RPC, Eq. 7; deterministic
// truncation).  Four packed token positions per lane; the 16 lanes of a 64-token
// group combine their bits into two 32-bit mask words.
#include "nat_internal.h"
#include "philox.hip.h"

namespace nat {

__global__ void advantage_kernel(const float* __restrict__ rewards, int P, int G, float eps_adv,
                                 float* __restrict__ adv) {
  // one wavefront per prompt; fixed-order lane-strided sums then a butterfly
  const int prompt = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (prompt >= P) return;
  const float* R = rewards + (size_t)prompt * G;
  float s = 0.f;
  for (int j = lane; j < G; j += 64) s += R[j];
  for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
  const float mu = s / (float)G;
  float q = 0.f;
  for (int j = lane; j < G; j += 64) { const float d = R[j] - mu; q += d * d; }
  for (int off = 32; off > 0; off >>= 1) q += __shfl_xor(q, off);
  const float sigma = sqrtf(q / (float)G);
  for (int j = lane; j < G; j += 64) adv[(size_t)prompt * G + j] = (R[j] - mu) / (sigma + eps_adv);
}

// cut_len[i] = L_i (RPC), K_i (DET), T_i (FULL, URS)
__global__ void select_cut_kernel(SelectArgs a, const int64_t* __restrict__ cu, int B,
                                  int32_t* __restrict__ cut_len) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= B) return;
  const int64_t T = cu[i + 1] - cu[i];
  const int scheme = a.scheme_per_rollout ? a.scheme_per_rollout[i] : a.scheme;
  int64_t cut = T;
  if (T > 0 && scheme == NAT_SCHEME_RPC) {
    int64_t Ci = a.min_cut < 1 ? 1 : a.min_cut;
    if (Ci > T) Ci = T;
    const uint64_t n = (uint64_t)(T - Ci + 1);
    const u32x4 r = philox4x32_10(u32x4{0u, (uint32_t)(a.rollout_id_base + i), 1u, a.step}, a.key0, a.key1);
    cut = Ci + (int64_t)(((uint64_t)r.x * n) >> 32);
  } else if (scheme == NAT_SCHEME_DET) {
    cut = (int64_t)floor(a.trunc_frac * (double)T);
  }
  if (a.drop_zero_adv && a.drop_zero_adv[i] == 0.f) cut = 0;
  cut_len[i] = (int32_t)cut;
}

// Four consecutive packed positions per lane: the four words of one Philox block serve four
// consecutive tokens of a rollout, so a lane evaluates one block (a second one where its
// positions straddle a block or rollout boundary) and one rollout search instead of four.
// A wavefront covers 256 positions = four 64-bit mask groups; the 16 lanes of a group OR
// their nibbles together and the group's first lane writes the two words.
constexpr int kSelPerLane = 4;
constexpr int kSelPerBlock = 256 * kSelPerLane;

__global__ void __launch_bounds__(256)
select_mask_kernel(SelectArgs a, const int64_t* __restrict__ cu, int B, int64_t N,
                   const int32_t* __restrict__ cut_len, uint32_t* __restrict__ mask_bits) {
  const int64_t n0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * kSelPerLane;
  uint32_t nibble = 0;
  // positions at or beyond cu[B] belong to no rollout (the host-passed N may be larger): never kept
  const int64_t n_end = cu[B] < N ? cu[B] : N;
  if (n0 < n_end) {
    int i = rollout_of_pos(cu, 0, B, n0);
    int64_t start = cu[i], end = cu[i + 1];
    int scheme = a.scheme_per_rollout ? a.scheme_per_rollout[i] : a.scheme;
    bool dropped = a.drop_zero_adv && a.drop_zero_adv[i] == 0.f;
    int64_t cut = cut_len[i];
    u32x4 r{0u, 0u, 0u, 0u};
    int64_t have_block = -1;                       // index (t0 >> 2) of the block held in r, for rollout i
#pragma unroll
    for (int j = 0; j < kSelPerLane; ++j) {
      const int64_t n = n0 + j;
      if (n >= n_end) break;
      if (n >= end) {                              // next non-empty rollout (n < cu[B]: one exists below B)
        do { ++i; } while (i < B - 1 && cu[i + 1] <= n);
        start = cu[i];
        end = cu[i + 1];
        scheme = a.scheme_per_rollout ? a.scheme_per_rollout[i] : a.scheme;
        dropped = a.drop_zero_adv && a.drop_zero_adv[i] == 0.f;
        cut = cut_len[i];
        have_block = -1;
      }
      const int64_t t0 = n - start;
      bool keep;
      if (scheme == NAT_SCHEME_URS) {
        if ((t0 >> 2) != have_block) {
          have_block = t0 >> 2;
          r = philox4x32_10(u32x4{(uint32_t)have_block, (uint32_t)(a.rollout_id_base + i), 0u, a.step}, a.key0, a.key1);
        }
        const uint32_t word = (t0 & 3) == 0 ? r.x : (t0 & 3) == 1 ? r.y : (t0 & 3) == 2 ? r.z : r.w;
        keep = (uint64_t)word < a.urs_threshold;
      } else if (scheme == NAT_SCHEME_FULL) {
        keep = true;
      } else {
        keep = t0 < cut;
      }
      if (keep && !dropped) nibble |= 1u << j;
    }
  }
  // lane l of a 16-lane group holds bits 4*(l%16) .. +3 of the group's 64-bit mask
  const int sub = threadIdx.x & 15;
  uint32_t lo = sub < 8 ? nibble << (4 * sub) : 0u;
  uint32_t hi = sub >= 8 ? nibble << (4 * (sub - 8)) : 0u;
#pragma unroll
  for (int off = 1; off < 16; off <<= 1) {
    lo |= __shfl_xor(lo, off);
    hi |= __shfl_xor(hi, off);
  }
  // groups past ceil(N/64) have no words in the mask
  if (sub == 0 && n0 < N) {
    const int64_t group = n0 >> 6;
    mask_bits[2 * group] = lo;
    mask_bits[2 * group + 1] = hi;
  }
}

nat_status validate_select(const nat_select_params* p, SelectArgs* out) {
  if (!p) return NAT_INVALID_ARG;
  if (p->scheme < NAT_SCHEME_FULL || p->scheme > NAT_SCHEME_DET) return NAT_INVALID_ARG;
  if (!(p->p > 0.0 && p->p <= 1.0)) return NAT_INVALID_ARG;
  if (p->min_cut < 1) return NAT_INVALID_ARG;
  if (!(p->trunc_frac > 0.0 && p->trunc_frac <= 1.0)) return NAT_INVALID_ARG;
  out->scheme = p->scheme;
  out->min_cut = p->min_cut;
  out->p = p->p;
  out->trunc_frac = p->trunc_frac;
  out->urs_threshold = (uint64_t)floor(p->p * 4294967296.0);
  out->key0 = (uint32_t)(p->seed & 0xFFFFFFFFull);
  out->key1 = (uint32_t)(p->seed >> 32);
  out->step = p->step;
  out->rollout_id_base = p->rollout_id_base;
  out->scheme_per_rollout = p->d_scheme_per_rollout;
  out->drop_zero_adv = p->d_drop_zero_adv;
  return NAT_OK;
}

nat_status launch_prefix_mask(const int64_t* d_cu, int32_t B, int64_t N, const int32_t* d_cut_len,
                              uint32_t* d_mask_bits, hipStream_t s) {
  if (N <= 0) return NAT_OK;
  SelectArgs a{};
  a.scheme = NAT_SCHEME_DET;        // any prefix scheme: keep t0 < cut_len[i]
  select_mask_kernel<<<(unsigned)((N + kSelPerBlock - 1) / kSelPerBlock), 256, 0, s>>>(a, d_cu, B, N, d_cut_len, d_mask_bits);
  NAT_LAUNCH_CHECK();
  return NAT_OK;
}

}  // namespace nat

using namespace nat;

extern "C" nat_status nat_advantage(const float* d_rewards, int32_t P, int32_t G, float eps_adv,
                                    float* d_adv, void* stream) {
  if (!d_rewards || !d_adv || P <= 0 || G <= 0 || !(eps_adv >= 0.f)) return NAT_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  ProfScope prof(PC_ADVANTAGE, s);
  const int waves_per_block = 4;
  advantage_kernel<<<(P + waves_per_block - 1) / waves_per_block, 64 * waves_per_block, 0, s>>>(
      d_rewards, P, G, eps_adv, d_adv);
  NAT_LAUNCH_CHECK();
  return NAT_OK;
}

extern "C" int64_t nat_mask_words(int64_t N) { return N <= 0 ? 0 : 2 * ((N + 63) / 64); }

extern "C" nat_status nat_select(const nat_select_params* params, const int64_t* d_cu_seqlens, int32_t B,
                                 int64_t N, int32_t* d_cut_len, uint32_t* d_mask_bits, void* stream) {
  SelectArgs a;
  nat_status st = validate_select(params, &a);
  if (st != NAT_OK) return st;
  if (!d_cu_seqlens || !d_cut_len || B <= 0 || N < 0 || N >= (int64_t(1) << 31)) return NAT_INVALID_ARG;
  if (N > 0 && !d_mask_bits) return NAT_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  ProfScope prof(PC_SELECT, s);
  select_cut_kernel<<<(B + 255) / 256, 256, 0, s>>>(a, d_cu_seqlens, B, d_cut_len);
  NAT_LAUNCH_CHECK();
  if (N > 0) {
    const int64_t blocks = (N + kSelPerBlock - 1) / kSelPerBlock;
    select_mask_kernel<<<(unsigned)blocks, 256, 0, s>>>(a, d_cu_seqlens, B, N, d_cut_len, d_mask_bits);
    NAT_LAUNCH_CHECK();
  }
  return NAT_OK;
}
