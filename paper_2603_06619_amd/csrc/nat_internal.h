// Internal declarations shared by the library's translation units (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "nat.h"

namespace nat {

// Kernel classes for the optional per-kernel timing.
enum ProfClass : int {
  PC_ADVANTAGE = 0, PC_SELECT, PC_COMPACT, PC_GATHER, PC_TRANSPOSE, PC_LOGITS, PC_TOKEN_STATS,
  PC_DHIDDEN, PC_DWEIGHT, PC_LOSS_REDUCE, PC_F32_PATH, PC_FILL, PC_SCHEDULE, PC_PREFIX_PACK, PC_NUM
};

// Brackets the launches issued during its lifetime with two events when timing is on.
struct ProfScope {
  ProfScope(int cls, hipStream_t s, bool enabled = true);
  ~ProfScope();
  int cls_; hipStream_t s_; void* rec_;
};

inline nat_status hip_status(hipError_t e) { return e == hipSuccess ? NAT_OK : NAT_HIP_ERROR; }
#define NAT_HIP_TRY(expr) do { hipError_t e__ = (expr); if (e__ != hipSuccess) return NAT_HIP_ERROR; } while (0)
#define NAT_LAUNCH_CHECK() do { hipError_t e__ = hipGetLastError(); if (e__ != hipSuccess) return NAT_HIP_ERROR; } while (0)

// Validated host-side copy of the selection parameters handed to kernels by value.
struct SelectArgs {
  int32_t scheme; int32_t min_cut; double p; double trunc_frac;
  uint64_t urs_threshold;       // floor(p * 2^32)
  uint32_t key0, key1, step; int32_t rollout_id_base;
  const int32_t* scheme_per_rollout;
  const float* drop_zero_adv;   // optional [B]: rollouts with advantage exactly 0 keep nothing
};
nat_status validate_select(const nat_select_params* p, SelectArgs* out);

// Rollout that contains packed position n: the last i in [lo, hi) with cu[i] <= n (skips
// empty rollouts, whose offsets repeat).  The caller guarantees cu[lo] <= n < cu[hi].
template <typename OffsetT>
__device__ __forceinline__ int rollout_of_pos(const OffsetT* __restrict__ cu, int lo, int hi, int64_t n) {
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if ((int64_t)cu[mid] <= n) lo = mid; else hi = mid;
  }
  return lo;
}

// mask bit n = (position of n inside its rollout) < cut_len[rollout]   (select.hip)
nat_status launch_prefix_mask(const int64_t* d_cu, int32_t B, int64_t N, const int32_t* d_cut_len,
                              uint32_t* d_mask_bits, hipStream_t s);

// nat_compact / nat_compact_pi share one implementation (compact.hip): weights come from
// the scheme's closed form when d_pi is NULL, else from the given probabilities.
struct CompactArgs {
  int32_t n_rollouts_global; const uint32_t* mask_bits; const double* pi; const int64_t* cu; int32_t B; int64_t N;
  int64_t kept_cap;             // capacity of the per-kept-token outputs
  int32_t* kept_idx; int32_t* kept_seq; float* kept_w; int32_t* cu_kept; int32_t* n_kept; int32_t* h_n_kept;
  const void* hidden; void* hidden_k; int32_t H; int32_t dtype;
  const int32_t* ids; int32_t* ids_k; const float* old_logp; float* old_logp_k;
  void* ws; size_t ws_bytes; hipStream_t stream;
  bool no_timing;               // never create timing events (the entry point that must not allocate)
};
nat_status compact_run(const SelectArgs& sel, const CompactArgs& c);

// bf16 loss path (loss_bf16.hip) and fp32 loss path (loss_f32.hip)
struct LossArgs {
  const void* hidden; const void* W; const int32_t* ids; const float* old_logp; const float* adv;
  const int32_t* kept_seq; const float* kept_w; int32_t N_k, H, V;
  float eps_lo, eps_hi, grad_scale;
  float* loss; float* logp; void* dH; float* dW; int32_t accumulate_dw;
  void* ws; size_t ws_bytes; hipStream_t stream;
  // KL term of Eq. 4 and the diagnostics of nat_loss_fwd_bwd_kl (all optional)
  const float* ref_logp; float beta_kl; int32_t kl_kind; float* kl_out; float* entropy_out;
  int32_t* diag;                // optional [NAT_DIAG_WORDS] counters, already cleared by the entry point
};
size_t loss_bf16_workspace_bytes(int32_t N_k, int32_t H, int32_t V, bool minimal);
nat_status loss_bf16_run(const LossArgs& a);
size_t loss_f32_workspace_bytes(int32_t N_k, int32_t H, int32_t V, bool minimal);
nat_status loss_f32_run(const LossArgs& a);

// forward pass alone (log-prob of given tokens, optional entropy)
struct LogpArgs {
  const void* hidden; const void* W; const int32_t* ids; int32_t N_k, H, V;
  float* logp; float* entropy; void* ws; size_t ws_bytes; hipStream_t stream;
  int32_t* diag;                // optional [NAT_DIAG_WORDS] counters, already cleared by the entry point
};
size_t logp_bf16_workspace_bytes(int32_t N_k, int32_t H, int32_t V, bool minimal);
nat_status logp_bf16_run(const LogpArgs& a);
size_t logp_f32_workspace_bytes(int32_t N_k, int32_t H, int32_t V, bool minimal);
nat_status logp_f32_run(const LogpArgs& a);

// shared small kernels (api.hip)
nat_status fill_zero_f32(float* p, size_t n, hipStream_t s);

// One atomic per wavefront: adds the number of lanes whose `flag` is set to *counter.  Every lane
// of the wavefront must call it (integer adds: the total does not depend on their order).
__device__ __forceinline__ void wave_count(bool flag, int32_t* counter) {
  const unsigned long long b = __ballot(flag);
  if (b != 0ull && (threadIdx.x & 63) == 0) atomicAdd(counter, (int32_t)__popcll(b));
}

}  // namespace nat
