// Per-token scalar part of the loss (Eq. 1, Eq. 3) and the fixed-order loss
// reduction, shared by the bf16 and fp32 paths.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "nat.h"

namespace nat {

// KL term of Eq. 4 (sampled-token forms; the footnote to Eq. 4 names the first).
struct KlArgs {
  const float* ref_logp;   // [N_k] log-probability of the sampled token under the reference policy
  float beta;              // 0 disables the term (ref_logp is then not read)
  int kind;                // NAT_KL_LOG_RATIO or NAT_KL_NONNEG
};

struct TokenScalars { float L; float c; float kl; bool clipped; };   // clipped: A != 0 and dS/dlogp = 0

// r = exp(logp - old_logp); S = min(r A, clip(r, 1-eps_lo, 1+eps_hi) A);
// dS/dlogp = r A on the unclipped branch (boundaries inclusive), else 0;
// with d = ref_logp - logp:  KL = -d (log-ratio form) or exp(d) - d - 1 (non-negative form),
// dKL/dlogp = 1 or 1 - exp(d);
// token objective L = S - beta KL;  c = dLoss/dlogp = -grad_scale * w * (dS/dlogp - beta dKL/dlogp).
__device__ __forceinline__ TokenScalars grpo_token_scalars(float logp, float old_logp, float A, float w,
                                                           float eps_lo, float eps_hi, float grad_scale,
                                                           float beta_kl, int kl_kind, float ref_logp) {
  const float r = expf(logp - old_logp);
  const float r_clip = fminf(fmaxf(r, 1.f - eps_lo), 1.f + eps_hi);
  const float S = fminf(r * A, r_clip * A);
  const bool active = (A > 0.f && r <= 1.f + eps_hi) || (A < 0.f && r >= 1.f - eps_lo);
  float g = active ? r * A : 0.f;
  TokenScalars out;
  out.clipped = A != 0.f && !active;
  out.L = S;
  out.kl = 0.f;
  if (beta_kl != 0.f) {
    const float d = ref_logp - logp;
    float kl, dkl;
    if (kl_kind == NAT_KL_NONNEG) {
      const float ed = expf(d);
      kl = ed - d - 1.f;
      dkl = 1.f - ed;
    } else {
      kl = -d;
      dkl = 1.f;
    }
    out.kl = kl;
    out.L = S - beta_kl * kl;
    g -= beta_kl * dkl;
  }
  out.c = -grad_scale * w * g;
  return out;
}

// loss = -sum_k term[k], one block, fixed order: lane-strided fp64 partial sums,
// then a fixed binary tree over the 1024 partials.
static __global__ void __launch_bounds__(1024)
loss_reduce_kernel(const float* __restrict__ term, int n, float* __restrict__ loss) {
  __shared__ double part[1024];
  double s = 0.0;
  for (int k = threadIdx.x; k < n; k += 1024) s += (double)term[k];
  part[threadIdx.x] = s;
  __syncthreads();
  for (int half = 512; half > 0; half >>= 1) {
    if ((int)threadIdx.x < half) part[threadIdx.x] += part[threadIdx.x + half];
    __syncthreads();
  }
  if (threadIdx.x == 0) *loss = (float)(-part[0]);
}

}  // namespace nat
