// nat_select_schedule: cut L_i drawn from an arbitrary cut-length distribution
// q_i given as integer weights, mask 1{t <= L_i} and survival function
// p_{i,t} = sum_{l >= t} q_i(l) (Sec. 4, Eq. 7-8).
// nat_select_poisson: independent Bernoulli(p_{i,t}) masks with caller-supplied
// probabilities (Sec. 3.1).
// nat_prefix_pack: the truncated batch (prompt + kept prefix per rollout) a model
// body needs to run only over kept prefixes (Sec. 4, forward truncation).
#include "nat_internal.h"
#include "philox.hip.h"

namespace nat {

constexpr int kSchedThreads = 256;

// Inclusive scan of one 64-bit value per thread over a 256-thread block; *total = block sum.
// `wave_tot` is 4 words of LDS; the caller separates successive calls with a barrier.
__device__ __forceinline__ uint64_t block_scan_u64(uint64_t v, uint64_t* wave_tot, uint64_t* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint64_t incl = v;
  for (int off = 1; off < 64; off <<= 1) {
    const uint64_t up = __shfl_up((unsigned long long)incl, off);
    if (lane >= off) incl += up;
  }
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  uint64_t before = 0, all = 0;
  for (int w = 0; w < kSchedThreads / 64; ++w) {
    const uint64_t t = wave_tot[w];
    if (w < wave) before += t;
    all += t;
  }
  *total = all;
  return before + incl;
}

// One block per rollout: total weight, the cut by inversion of the running sum, and the
// survival function for every position.
__global__ void __launch_bounds__(kSchedThreads)
schedule_cut_kernel(uint32_t key0, uint32_t key1, uint32_t step, int32_t rollout_id_base,
                    const float* __restrict__ drop_zero_adv,
                    const uint32_t* __restrict__ weights, const int64_t* __restrict__ cu, int64_t N,
                    int32_t* __restrict__ cut_len, double* __restrict__ pi) {
  __shared__ uint64_t wave_tot[kSchedThreads / 64];
  const int i = blockIdx.x;
  // offsets are clamped to the N positions the caller's arrays hold
  const int64_t start = cu[i] < 0 ? 0 : cu[i] > N ? N : cu[i];
  const int64_t stop = cu[i + 1] > N ? N : cu[i + 1];
  const int64_t T = stop - start;
  if (T <= 0) {
    if (threadIdx.x == 0) cut_len[i] = 0;
    return;
  }
  const uint32_t* a = weights + start;
  double* p = pi + start;

  uint64_t part = 0;
  for (int64_t j = threadIdx.x; j < T; j += kSchedThreads) part += a[j];
  uint64_t A;
  block_scan_u64(part, wave_tot, &A);
  __syncthreads();
  if (A == 0) {                                   // no schedule: keep the rollout whole, p = 1
    for (int64_t j = threadIdx.x; j < T; j += kSchedThreads) p[j] = 1.0;
    if (threadIdx.x == 0) cut_len[i] = (drop_zero_adv && drop_zero_adv[i] == 0.f) ? 0 : (int32_t)T;
    return;
  }
  const u32x4 rnd = philox4x32_10(u32x4{0u, (uint32_t)(rollout_id_base + i), 2u, step}, key0, key1);
  uint64_t r = __umul64hi(((uint64_t)rnd.x << 32) | (uint64_t)rnd.y, A);         // in [0, A)
  const bool dropped = drop_zero_adv && drop_zero_adv[i] == 0.f;                 // keeps nothing: no position
  if (dropped) {                                                                 // qualifies below
    r = ~0ull;
    if (threadIdx.x == 0) cut_len[i] = 0;
  }

  const double den = (double)A;
  uint64_t carry = 0;                              // running sum of all earlier positions
  constexpr int kPer = 4;                          // consecutive positions per thread and iteration
  for (int64_t base = 0; base < T; base += kSchedThreads * kPer) {
    const int64_t j0 = base + (int64_t)threadIdx.x * kPer;
    uint32_t v[kPer];
    uint64_t mine = 0;
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
      v[e] = j0 + e < T ? a[j0 + e] : 0u;
      mine += v[e];
    }
    uint64_t chunk_total;
    uint64_t run = carry + block_scan_u64(mine, wave_tot, &chunk_total) - mine;   // sum of positions before j0
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
      if (j0 + e < T) {
        p[j0 + e] = (double)(A - run) / den;      // sum_{l >= t} a_l over A, exact integers below 2^53
        if (run <= r && r < run + v[e]) cut_len[i] = (int32_t)(j0 + e + 1);   // exactly one position qualifies
      }
      run += v[e];
    }
    carry += chunk_total;
    __syncthreads();
  }
}

// Four consecutive packed positions per lane (one Philox block serves four consecutive tokens of a
// rollout); the 16 lanes of a 64-token group OR their nibbles into the two mask words.
__global__ void __launch_bounds__(256)
poisson_mask_kernel(uint32_t key0, uint32_t key1, uint32_t step, int32_t rollout_id_base,
                    const float* __restrict__ drop_zero_adv, const double* __restrict__ pi,
                    const int64_t* __restrict__ cu, int B, int64_t N, uint32_t* __restrict__ mask_bits) {
  const int64_t n0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  uint32_t nibble = 0;
  const int64_t n_end = cu[B] < N ? cu[B] : N;     // positions beyond the last rollout are never kept
  if (n0 < n_end) {
    int i = rollout_of_pos(cu, 0, B, n0);
    int64_t start = cu[i], end = cu[i + 1];
    bool dropped = drop_zero_adv && drop_zero_adv[i] == 0.f;
    u32x4 r{0u, 0u, 0u, 0u};
    int64_t have_block = -1;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t n = n0 + j;
      if (n >= n_end) break;
      if (n >= end) {
        do { ++i; } while (i < B - 1 && cu[i + 1] <= n);
        start = cu[i];
        end = cu[i + 1];
        dropped = drop_zero_adv && drop_zero_adv[i] == 0.f;
        have_block = -1;
      }
      const int64_t t0 = n - start;
      if ((t0 >> 2) != have_block) {
        have_block = t0 >> 2;
        r = philox4x32_10(u32x4{(uint32_t)have_block, (uint32_t)(rollout_id_base + i), 0u, step}, key0, key1);
      }
      const double p = pi[n];
      uint64_t thr = 0;                                           // p <= 0 or NaN: never keep
      if (p >= 1.0) thr = 1ull << 32;
      else if (p > 0.0) thr = (uint64_t)floor(p * 4294967296.0);
      const uint32_t word = (t0 & 3) == 0 ? r.x : (t0 & 3) == 1 ? r.y : (t0 & 3) == 2 ? r.z : r.w;
      if ((uint64_t)word < thr && !dropped) nibble |= 1u << j;
    }
  }
  const int sub = threadIdx.x & 15;
  uint32_t lo = sub < 8 ? nibble << (4 * sub) : 0u;
  uint32_t hi = sub >= 8 ? nibble << (4 * (sub - 8)) : 0u;
#pragma unroll
  for (int off = 1; off < 16; off <<= 1) {
    lo |= __shfl_xor(lo, off);
    hi |= __shfl_xor(hi, off);
  }
  if (sub == 0 && n0 < N) {
    const int64_t group = n0 >> 6;
    mask_bits[2 * group] = lo;
    mask_bits[2 * group + 1] = hi;
  }
}

// cu_packed = exclusive scan of P_i + L_i, cu_loss = exclusive scan of L_i, totals = (rows, longest).
__global__ void __launch_bounds__(1024)
prefix_scan_kernel(const int32_t* __restrict__ prompt_len, const int64_t* __restrict__ cu,
                   const int32_t* __restrict__ cut_len, int B, int32_t* __restrict__ cu_packed,
                   int32_t* __restrict__ cu_loss, int32_t* __restrict__ totals) {
  __shared__ int wave_rows[16], wave_loss[16], wave_max[16];
  __shared__ int carry_rows, carry_loss;
  if (threadIdx.x == 0) { carry_rows = 0; carry_loss = 0; }
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int longest = 0;
  for (int base = 0; base < B; base += 1024) {
    const int i = base + threadIdx.x;
    int L = 0, rows = 0;
    if (i < B) {
      const int64_t T = cu[i + 1] - cu[i];
      const int64_t c = cut_len[i];
      L = (int)(c < 0 ? 0 : c > T ? T : c);
      rows = (prompt_len ? prompt_len[i] : 0) + L;
      longest = rows > longest ? rows : longest;
    }
    int in_rows = rows, in_loss = L;
    for (int off = 1; off < 64; off <<= 1) {
      const int ur = __shfl_up(in_rows, off), ul = __shfl_up(in_loss, off);
      if (lane >= off) { in_rows += ur; in_loss += ul; }
    }
    if (lane == 63) { wave_rows[wave] = in_rows; wave_loss[wave] = in_loss; }
    __syncthreads();
    int before_rows = carry_rows, before_loss = carry_loss;
    for (int w = 0; w < wave; ++w) { before_rows += wave_rows[w]; before_loss += wave_loss[w]; }
    if (i < B) { cu_packed[i] = before_rows + in_rows - rows; cu_loss[i] = before_loss + in_loss - L; }
    __syncthreads();
    if (threadIdx.x == 1023) { carry_rows = before_rows + in_rows; carry_loss = before_loss + in_loss; }
    __syncthreads();
  }
  for (int off = 32; off > 0; off >>= 1) { const int o = __shfl_xor(longest, off); longest = o > longest ? o : longest; }
  if (lane == 0) wave_max[wave] = longest;
  __syncthreads();
  if (threadIdx.x == 0) {
    int m = 0;
    for (int w = 0; w < 16; ++w) m = wave_max[w] > m ? wave_max[w] : m;
    cu_packed[B] = carry_rows;
    cu_loss[B] = carry_loss;
    totals[0] = carry_rows;
    totals[1] = m;
  }
}

// One lane per row of the truncated batch.
__global__ void __launch_bounds__(256)
prefix_rows_kernel(const int32_t* __restrict__ prompt_len, const int64_t* __restrict__ cu, int B, int shift,
                   int64_t rows_cap, int64_t kept_cap, const int32_t* __restrict__ cu_packed,
                   const int32_t* __restrict__ cu_loss, int32_t* __restrict__ src_idx,
                   int32_t* __restrict__ position_ids, int32_t* __restrict__ loss_row,
                   const int32_t* __restrict__ input_ids, int32_t* __restrict__ input_ids_packed) {
  const int64_t m = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (m >= rows_cap || m >= (int64_t)cu_packed[B]) return;
  const int i = rollout_of_pos(cu_packed, 0, B, m);
  const int j = (int)(m - cu_packed[i]);
  const int P = prompt_len ? prompt_len[i] : 0;
  // rows of the full input before rollout i: all earlier prompts and all earlier full responses
  const int64_t full_start = (int64_t)(cu_packed[i] - cu_loss[i]) + cu[i];
  const int64_t src = full_start + j;
  src_idx[m] = (int32_t)src;
  position_ids[m] = j;
  if (input_ids) input_ids_packed[m] = input_ids[src];
  if (j >= P) {
    const int64_t k = (int64_t)cu_loss[i] + (j - P);
    if (k < kept_cap) loss_row[k] = (int32_t)(m - shift);
  }
}

}  // namespace nat

using namespace nat;

static nat_status check_common(const nat_select_params* params, const void* a, const int64_t* cu, int32_t B,
                               int64_t N) {
  if (!params || !cu || B <= 0 || N < 0 || N >= (int64_t(1) << 31)) return NAT_INVALID_ARG;
  if (N > 0 && !a) return NAT_INVALID_ARG;
  return NAT_OK;
}

extern "C" nat_status nat_select_schedule(const nat_select_params* params, const uint32_t* d_weights,
                                          const int64_t* d_cu_seqlens, int32_t B, int64_t N,
                                          int32_t* d_cut_len, uint32_t* d_mask_bits, double* d_pi, void* stream) {
  nat_status st = check_common(params, d_weights, d_cu_seqlens, B, N);
  if (st != NAT_OK) return st;
  if (!d_cut_len || (N > 0 && (!d_mask_bits || !d_pi))) return NAT_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  ProfScope prof(PC_SCHEDULE, s);
  schedule_cut_kernel<<<(unsigned)B, kSchedThreads, 0, s>>>(
      (uint32_t)(params->seed & 0xFFFFFFFFull), (uint32_t)(params->seed >> 32), params->step,
      params->rollout_id_base, params->d_drop_zero_adv, d_weights, d_cu_seqlens, N, d_cut_len, d_pi);
  NAT_LAUNCH_CHECK();
  return launch_prefix_mask(d_cu_seqlens, B, N, d_cut_len, d_mask_bits, s);
}

extern "C" nat_status nat_select_poisson(const nat_select_params* params, const double* d_pi,
                                         const int64_t* d_cu_seqlens, int32_t B, int64_t N,
                                         uint32_t* d_mask_bits, void* stream) {
  nat_status st = check_common(params, d_pi, d_cu_seqlens, B, N);
  if (st != NAT_OK) return st;
  if (N > 0 && !d_mask_bits) return NAT_INVALID_ARG;
  if (N == 0) return NAT_OK;
  hipStream_t s = (hipStream_t)stream;
  ProfScope prof(PC_SCHEDULE, s);
  poisson_mask_kernel<<<(unsigned)((N + 1023) / 1024), 256, 0, s>>>(
      (uint32_t)(params->seed & 0xFFFFFFFFull), (uint32_t)(params->seed >> 32), params->step,
      params->rollout_id_base, params->d_drop_zero_adv, d_pi, d_cu_seqlens, B, N, d_mask_bits);
  NAT_LAUNCH_CHECK();
  return NAT_OK;
}

extern "C" nat_status nat_prefix_pack(const int32_t* d_prompt_len, const int64_t* d_cu_seqlens,
                                      const int32_t* d_cut_len, int32_t B, int32_t next_token_shift,
                                      int64_t rows_cap, int64_t kept_cap,
                                      int32_t* d_cu_packed, int32_t* d_cu_loss, int32_t* d_src_idx,
                                      int32_t* d_position_ids, int32_t* d_loss_row, int32_t* d_totals,
                                      int32_t* h_totals, const int32_t* d_input_ids,
                                      int32_t* d_input_ids_packed, void* stream) {
  if (!d_cu_seqlens || !d_cut_len || !d_cu_packed || !d_cu_loss || !d_totals || B <= 0 || rows_cap < 0 ||
      kept_cap < 0 || rows_cap >= (int64_t(1) << 31) || kept_cap >= (int64_t(1) << 31))
    return NAT_INVALID_ARG;
  if (next_token_shift != 0 && next_token_shift != 1) return NAT_INVALID_ARG;
  if (next_token_shift == 1 && !d_prompt_len) return NAT_INVALID_ARG;
  if (rows_cap > 0 && (!d_src_idx || !d_position_ids)) return NAT_INVALID_ARG;
  if (rows_cap > 0 && kept_cap > 0 && !d_loss_row) return NAT_INVALID_ARG;
  if ((d_input_ids != nullptr) != (d_input_ids_packed != nullptr)) return NAT_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  {
    ProfScope prof(PC_PREFIX_PACK, s);
    prefix_scan_kernel<<<1, 1024, 0, s>>>(d_prompt_len, d_cu_seqlens, d_cut_len, B, d_cu_packed, d_cu_loss, d_totals);
    NAT_LAUNCH_CHECK();
    if (rows_cap > 0) {
      prefix_rows_kernel<<<(unsigned)((rows_cap + 255) / 256), 256, 0, s>>>(
          d_prompt_len, d_cu_seqlens, B, next_token_shift, rows_cap, kept_cap, d_cu_packed, d_cu_loss, d_src_idx,
          d_position_ids, d_loss_row, d_input_ids, d_input_ids_packed);
      NAT_LAUNCH_CHECK();
    }
  }
  if (h_totals) NAT_HIP_TRY(hipMemcpyAsync(h_totals, d_totals, 2 * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  return NAT_OK;
}
