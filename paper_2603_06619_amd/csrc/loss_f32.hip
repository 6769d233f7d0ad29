// fp32 path of nat_loss_fwd_bwd (small heads: the tiny fp32 workload).  Plain
// vector-ALU kernels, fixed summation order, one token chunk at a time:
//   forward   one block per token: z = W h (one wavefront per vocabulary row),
//             log-sum-exp, log-prob of the target, ratio / clipped surrogate
//             (Eq. 1, Eq. 3), then dz = c (onehot - softmax) in the chunk scratch;
//   dH        dH_k = sum_v dz_kv W_v       (one block per token, lanes over H);
//   dW        dW_v += sum_k dz_kv h_k      (one thread per (v, h), tokens in order).
#include "nat_internal.h"
#include "grpo_scalar.hip.h"

namespace nat {

constexpr int kF32Threads = 256;

__device__ __forceinline__ float wave_sum_f(float v) {
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
}
__device__ __forceinline__ float wave_max_f(float v) {
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  return v;
}

__global__ void __launch_bounds__(kF32Threads)
f32_forward_kernel(const float* __restrict__ hidden, const float* __restrict__ W, const int32_t* __restrict__ ids,
                   const float* __restrict__ old_logp, const float* __restrict__ adv,
                   const int32_t* __restrict__ kept_seq, const float* __restrict__ kept_w,
                   int chunk_start, int H, int V, float eps_lo, float eps_hi, float grad_scale, KlArgs klp,
                   float* __restrict__ dz /*[chunk, V]*/, float* __restrict__ logp_out, float* __restrict__ term,
                   float* __restrict__ kl_out, float* __restrict__ entropy_out, int32_t* __restrict__ diag) {
  extern __shared__ float h_s[];             // H floats
  __shared__ float red[4];
  __shared__ float bcast[2];
  const int kc = blockIdx.x;                 // token within the chunk
  const int k = chunk_start + kc;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int h = threadIdx.x; h < H; h += kF32Threads) h_s[h] = hidden[(size_t)k * H + h];
  __syncthreads();
  float* z = dz + (size_t)kc * V;
  for (int v = wave; v < V; v += 4) {
    const float* wr = W + (size_t)v * H;
    float p = 0.f;
    for (int h = lane; h < H; h += 64) p = fmaf(wr[h], h_s[h], p);
    p = wave_sum_f(p);
    if (lane == 0) z[v] = p;
  }
  __syncthreads();
  float m = -INFINITY;
  for (int v = threadIdx.x; v < V; v += kF32Threads) m = fmaxf(m, z[v]);
  m = wave_max_f(m);
  if (lane == 0) red[wave] = m;
  __syncthreads();
  m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float s = 0.f, t = 0.f;                    // sum of e^(z-m) and of e^(z-m) (z-m)
  for (int v = threadIdx.x; v < V; v += kF32Threads) {
    const float zc = z[v] - m, e = expf(zc);
    s += e;
    t = fmaf(e, zc, t);
  }
  s = wave_sum_f(s);
  t = wave_sum_f(t);
  __shared__ float red_t[4];
  if (lane == 0) { red[wave] = s; red_t[wave] = t; }
  __syncthreads();
  if (threadIdx.x == 0) {
    const float sum = (red[0] + red[1]) + (red[2] + red[3]);
    const float lse = m + logf(sum);
    // -sum p log p = log(sum) - (sum of e (z - m)) / sum
    if (entropy_out) entropy_out[k] = logf(sum) - ((red_t[0] + red_t[1]) + (red_t[2] + red_t[3])) / sum;
    const int yk = ids[k];
    bcast[0] = lse;
    if (yk < 0 || yk >= V) {                 // no such token: left out (no loss term, zero gradient)
      if (logp_out) logp_out[k] = __builtin_nanf("");
      if (kl_out) kl_out[k] = __builtin_nanf("");
      term[k] = 0.f;
      bcast[1] = 0.f;
      if (diag) atomicAdd(diag + NAT_DIAG_BAD_ID, 1);
    } else {
      const float logp = z[yk] - lse;
      const float w = kept_w[k];
      const float A = adv[kept_seq[k]];
      const TokenScalars ts = grpo_token_scalars(logp, old_logp[k], A, w, eps_lo, eps_hi, grad_scale,
                                                 klp.beta, klp.kind, klp.beta != 0.f ? klp.ref_logp[k] : 0.f);
      if (logp_out) logp_out[k] = logp;
      if (kl_out) kl_out[k] = ts.kl;
      term[k] = w * ts.L;
      bcast[1] = ts.c;
      if (diag) {
        if (ts.clipped) atomicAdd(diag + NAT_DIAG_CLIPPED, 1);
        if (A != 0.f) atomicAdd(diag + NAT_DIAG_NONZERO_ADV, 1);
      }
    }
  }
  __syncthreads();
  const float lse = bcast[0], c = bcast[1];
  const int y = ids[k];
  for (int v = threadIdx.x; v < V; v += kF32Threads) {
    const float sm = expf(z[v] - lse);
    z[v] = c * ((v == y ? 1.f : 0.f) - sm);
  }
}

__global__ void __launch_bounds__(kF32Threads)
f32_dh_kernel(const float* __restrict__ dz, const float* __restrict__ W, int chunk_start, int H, int V,
              float* __restrict__ dH) {
  const int kc = blockIdx.x;
  const float* d = dz + (size_t)kc * V;
  for (int h = threadIdx.x; h < H; h += kF32Threads) {
    float acc = 0.f;
    for (int v = 0; v < V; ++v) acc = fmaf(d[v], W[(size_t)v * H + h], acc);
    dH[(size_t)(chunk_start + kc) * H + h] = acc;
  }
}

__global__ void __launch_bounds__(kF32Threads)
f32_dw_kernel(const float* __restrict__ dz, const float* __restrict__ hidden, int chunk_start, int chunk_n,
              int H, int V, int accumulate, float* __restrict__ dW) {
  const int v = blockIdx.x;
  for (int h = blockIdx.y * kF32Threads + threadIdx.x; h < H; h += gridDim.y * kF32Threads) {
    float acc = accumulate ? dW[(size_t)v * H + h] : 0.f;
    for (int kc = 0; kc < chunk_n; ++kc)
      acc = fmaf(dz[(size_t)kc * V + v], hidden[(size_t)(chunk_start + kc) * H + h], acc);
    dW[(size_t)v * H + h] = acc;
  }
}

static int f32_chunk_rows(int32_t N_k, int32_t V, size_t ws_bytes) {
  const size_t fixed = (size_t)N_k * sizeof(float) + 256;
  if (ws_bytes <= fixed) return 0;
  size_t rows = (ws_bytes - fixed) / ((size_t)V * sizeof(float));
  if (rows > (size_t)N_k) rows = N_k;
  return (int)rows;
}

size_t loss_f32_workspace_bytes(int32_t N_k, int32_t H, int32_t V, bool minimal) {
  (void)H;
  int rows = N_k < 1 ? 1 : N_k;
  const int cap = minimal ? 1 : 4096;
  if (rows > cap) rows = cap;
  return (size_t)N_k * sizeof(float) + 256 + (size_t)rows * V * sizeof(float);
}

nat_status loss_f32_run(const LossArgs& a) {
  if ((size_t)a.H * sizeof(float) > 60 * 1024) return NAT_BAD_SHAPE;      // h_k is staged in LDS
  const int rows = f32_chunk_rows(a.N_k, a.V, a.ws_bytes);
  if (rows < 1) return NAT_WORKSPACE_TOO_SMALL;
  float* term = (float*)a.ws;
  float* dz = (float*)((char*)a.ws + (((size_t)a.N_k * sizeof(float) + 255) / 256) * 256);
  hipStream_t s = a.stream;
  {
    ProfScope prof(PC_F32_PATH, s);
    for (int c0 = 0; c0 < a.N_k; c0 += rows) {
      const int n = a.N_k - c0 < rows ? a.N_k - c0 : rows;
      f32_forward_kernel<<<n, kF32Threads, (size_t)a.H * sizeof(float), s>>>(
          (const float*)a.hidden, (const float*)a.W, a.ids, a.old_logp, a.adv, a.kept_seq, a.kept_w, c0, a.H, a.V,
          a.eps_lo, a.eps_hi, a.grad_scale, KlArgs{a.ref_logp, a.beta_kl, a.kl_kind}, dz, a.logp, term,
          a.kl_out, a.entropy_out, a.diag);
      NAT_LAUNCH_CHECK();
      f32_dh_kernel<<<n, kF32Threads, 0, s>>>(dz, (const float*)a.W, c0, a.H, a.V, (float*)a.dH);
      NAT_LAUNCH_CHECK();
      const int gy = (a.H + kF32Threads - 1) / kF32Threads;
      f32_dw_kernel<<<dim3(a.V, gy > 64 ? 64 : gy), kF32Threads, 0, s>>>(
          dz, (const float*)a.hidden, c0, n, a.H, a.V, (c0 > 0 || a.accumulate_dw) ? 1 : 0, a.dW);
      NAT_LAUNCH_CHECK();
    }
  }
  ProfScope prof(PC_LOSS_REDUCE, s);
  loss_reduce_kernel<<<1, 1024, 0, s>>>(term, a.N_k, a.loss);
  NAT_LAUNCH_CHECK();
  return NAT_OK;
}


// Forward pass alone on the fp32 path: one block per token, logits kept in LDS-sized pieces of the
// chunk scratch, log-sum-exp with the true row maximum, entropy from the same two sums.
__global__ void __launch_bounds__(kF32Threads)
f32_logp_kernel(const float* __restrict__ hidden, const float* __restrict__ W, const int32_t* __restrict__ ids,
                int chunk_start, int H, int V, float* __restrict__ z_scratch /*[chunk, V]*/,
                float* __restrict__ logp_out, float* __restrict__ entropy_out, int32_t* __restrict__ diag) {
  extern __shared__ float h_s[];
  __shared__ float red[4], red_t[4];
  const int kc = blockIdx.x, k = chunk_start + kc;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int h = threadIdx.x; h < H; h += kF32Threads) h_s[h] = hidden[(size_t)k * H + h];
  __syncthreads();
  float* z = z_scratch + (size_t)kc * V;
  for (int v = wave; v < V; v += 4) {
    const float* wr = W + (size_t)v * H;
    float p = 0.f;
    for (int h = lane; h < H; h += 64) p = fmaf(wr[h], h_s[h], p);
    p = wave_sum_f(p);
    if (lane == 0) z[v] = p;
  }
  __syncthreads();
  float m = -INFINITY;
  for (int v = threadIdx.x; v < V; v += kF32Threads) m = fmaxf(m, z[v]);
  m = wave_max_f(m);
  if (lane == 0) red[wave] = m;
  __syncthreads();
  m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float s = 0.f, t = 0.f;
  for (int v = threadIdx.x; v < V; v += kF32Threads) {
    const float zc = z[v] - m, e = expf(zc);
    s += e;
    t = fmaf(e, zc, t);
  }
  s = wave_sum_f(s);
  t = wave_sum_f(t);
  if (lane == 0) { red[wave] = s; red_t[wave] = t; }
  __syncthreads();
  if (threadIdx.x == 0) {
    const float sum = (red[0] + red[1]) + (red[2] + red[3]);
    const int yk = ids[k];
    if (yk < 0 || yk >= V) {
      logp_out[k] = __builtin_nanf("");
      if (diag) atomicAdd(diag + NAT_DIAG_BAD_ID, 1);
    } else {
      logp_out[k] = z[yk] - (m + logf(sum));
    }
    if (entropy_out) entropy_out[k] = logf(sum) - ((red_t[0] + red_t[1]) + (red_t[2] + red_t[3])) / sum;
  }
}

size_t logp_f32_workspace_bytes(int32_t N_k, int32_t H, int32_t V, bool minimal) {
  (void)H;
  int rows = N_k < 1 ? 1 : N_k;
  const int cap = minimal ? 1 : 4096;
  if (rows > cap) rows = cap;
  return 256 + (size_t)rows * V * sizeof(float);
}

nat_status logp_f32_run(const LogpArgs& a) {
  if ((size_t)a.H * sizeof(float) > 60 * 1024) return NAT_BAD_SHAPE;
  if (a.ws_bytes < 256 + (size_t)a.V * sizeof(float)) return NAT_WORKSPACE_TOO_SMALL;
  size_t rows = (a.ws_bytes - 256) / ((size_t)a.V * sizeof(float));
  if (rows > (size_t)a.N_k) rows = a.N_k;
  hipStream_t s = a.stream;
  ProfScope prof(PC_F32_PATH, s);
  for (int c0 = 0; c0 < a.N_k; c0 += (int)rows) {
    const int n = a.N_k - c0 < (int)rows ? a.N_k - c0 : (int)rows;
    f32_logp_kernel<<<n, kF32Threads, (size_t)a.H * sizeof(float), s>>>(
        (const float*)a.hidden, (const float*)a.W, a.ids, c0, a.H, a.V, (float*)a.ws, a.logp, a.entropy, a.diag);
    NAT_LAUNCH_CHECK();
  }
  return NAT_OK;
}

}  // namespace nat
