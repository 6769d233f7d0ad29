// Status strings, the optional per-kernel event timing, small shared kernels and
// the nat_loss_fwd_bwd entry point (argument checks + dispatch by dtype).
#include "nat_internal.h"

#include <mutex>
#include <vector>

namespace nat {

namespace {
struct EventPair { hipEvent_t start, stop; int cls; };
std::mutex g_prof_mutex;
bool g_prof_on = false;
std::vector<EventPair> g_prof_records;
const char* const kClassNames[PC_NUM] = {
    "advantage", "select", "compact", "gather", "transpose", "logits_gemm", "token_stats",
    "dhidden_gemm", "dweight_gemm", "loss_reduce", "f32_path", "fill", "schedule", "prefix_pack"};
}  // namespace

ProfScope::ProfScope(int cls, hipStream_t s, bool enabled) : cls_(cls), s_(s), rec_(nullptr) {
  if (!enabled) return;
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  if (!g_prof_on) return;
  EventPair* ep = new EventPair{nullptr, nullptr, cls};
  if (hipEventCreate(&ep->start) != hipSuccess || hipEventCreate(&ep->stop) != hipSuccess ||
      hipEventRecord(ep->start, s) != hipSuccess) {
    delete ep;
    return;
  }
  rec_ = ep;
}

ProfScope::~ProfScope() {
  if (!rec_) return;
  EventPair* ep = (EventPair*)rec_;
  (void)hipEventRecord(ep->stop, s_);
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  g_prof_records.push_back(*ep);
  delete ep;
}

__global__ void fill_zero_kernel(float4* __restrict__ p4, size_t n4, float* __restrict__ tail, int n_tail) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride)
    p4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  if (blockIdx.x == 0 && (int)threadIdx.x < n_tail) tail[threadIdx.x] = 0.f;
}

nat_status fill_zero_f32(float* p, size_t n, hipStream_t s) {
  if (n == 0) return NAT_OK;
  ProfScope prof(PC_FILL, s);
  const size_t n4 = n / 4;
  size_t blocks = (n4 + 255) / 256;
  if (blocks > 8192) blocks = 8192;
  if (blocks == 0) blocks = 1;
  fill_zero_kernel<<<(unsigned)blocks, 256, 0, s>>>((float4*)p, n4, p + 4 * n4, (int)(n - 4 * n4));
  NAT_LAUNCH_CHECK();
  return NAT_OK;
}

}  // namespace nat

using namespace nat;

extern "C" const char* nat_status_string(nat_status s) {
  switch (s) {
    case NAT_OK: return "NAT_OK";
    case NAT_INVALID_ARG: return "NAT_INVALID_ARG";
    case NAT_BAD_SHAPE: return "NAT_BAD_SHAPE";
    case NAT_WORKSPACE_TOO_SMALL: return "NAT_WORKSPACE_TOO_SMALL";
    case NAT_UNSUPPORTED_DTYPE: return "NAT_UNSUPPORTED_DTYPE";
    case NAT_HIP_ERROR: return "NAT_HIP_ERROR";
    default: return "NAT_UNKNOWN_STATUS";
  }
}

extern "C" int32_t nat_profile_num_classes(void) { return PC_NUM; }

extern "C" const char* nat_profile_class_name(int32_t cls) {
  return (cls >= 0 && cls < PC_NUM) ? kClassNames[cls] : "unknown";
}

extern "C" nat_status nat_profile_enable(int32_t on) {
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  g_prof_on = on != 0;
  return NAT_OK;
}

extern "C" nat_status nat_profile_collect(double* h_ms, int64_t* h_launches, int32_t n_classes) {
  if (!h_ms || !h_launches || n_classes < PC_NUM) return NAT_INVALID_ARG;
  std::vector<EventPair> recs;
  {
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    recs.swap(g_prof_records);
  }
  nat_status st = NAT_OK;
  for (EventPair& ep : recs) {
    float ms = 0.f;
    if (hipEventSynchronize(ep.stop) != hipSuccess || hipEventElapsedTime(&ms, ep.start, ep.stop) != hipSuccess) {
      st = NAT_HIP_ERROR;
    } else {
      h_ms[ep.cls] += (double)ms;
      h_launches[ep.cls] += 1;
    }
    (void)hipEventDestroy(ep.start);
    (void)hipEventDestroy(ep.stop);
  }
  return st;
}

extern "C" size_t nat_loss_workspace_bytes(int32_t N_k, int32_t H, int32_t V, int32_t dtype) {
  if (N_k < 0 || H <= 0 || V <= 0) return 0;
  if (dtype == NAT_DTYPE_BF16) return (H % 64) ? 0 : loss_bf16_workspace_bytes(N_k, H, V, false);
  if (dtype == NAT_DTYPE_F32) return loss_f32_workspace_bytes(N_k, H, V, false);
  return 0;
}

extern "C" size_t nat_loss_workspace_min_bytes(int32_t N_k, int32_t H, int32_t V, int32_t dtype) {
  if (N_k < 0 || H <= 0 || V <= 0) return 0;
  if (dtype == NAT_DTYPE_BF16) return (H % 64) ? 0 : loss_bf16_workspace_bytes(N_k, H, V, true);
  if (dtype == NAT_DTYPE_F32) return loss_f32_workspace_bytes(N_k, H, V, true);
  return 0;
}

extern "C" size_t nat_logp_workspace_bytes(int32_t N_k, int32_t H, int32_t V, int32_t dtype) {
  if (N_k < 0 || H <= 0 || V <= 0) return 0;
  if (dtype == NAT_DTYPE_BF16) return (H % 64) ? 0 : logp_bf16_workspace_bytes(N_k, H, V, false);
  if (dtype == NAT_DTYPE_F32) return logp_f32_workspace_bytes(N_k, H, V, false);
  return 0;
}

extern "C" size_t nat_logp_workspace_min_bytes(int32_t N_k, int32_t H, int32_t V, int32_t dtype) {
  if (N_k < 0 || H <= 0 || V <= 0) return 0;
  if (dtype == NAT_DTYPE_BF16) return (H % 64) ? 0 : logp_bf16_workspace_bytes(N_k, H, V, true);
  if (dtype == NAT_DTYPE_F32) return logp_f32_workspace_bytes(N_k, H, V, true);
  return 0;
}

// the diagnostic counters are integers: cleared through the float fill (all-zero bits)
static nat_status clear_diag(int32_t* d_diag, hipStream_t s) {
  return d_diag ? fill_zero_f32((float*)d_diag, NAT_DIAG_WORDS, s) : NAT_OK;
}

extern "C" nat_status nat_logp_fwd(const void* d_hidden_k, const void* d_W, const int32_t* d_ids_k,
                                   int32_t N_k, int32_t H, int32_t V, int32_t dtype,
                                   float* d_logp_k, float* d_entropy_k, int32_t* d_diag,
                                   void* d_ws, size_t ws_bytes, void* stream) {
  if (dtype != NAT_DTYPE_F32 && dtype != NAT_DTYPE_BF16) return NAT_UNSUPPORTED_DTYPE;
  if (N_k < 0) return NAT_INVALID_ARG;
  if (H <= 0 || V <= 0) return NAT_BAD_SHAPE;
  if (dtype == NAT_DTYPE_BF16 && (H % 64) != 0) return NAT_BAD_SHAPE;
  if (N_k == 0) return clear_diag(d_diag, (hipStream_t)stream);
  if (!d_hidden_k || !d_W || !d_ids_k || !d_logp_k) return NAT_INVALID_ARG;
  if (!d_ws || ws_bytes < nat_logp_workspace_min_bytes(N_k, H, V, dtype)) return NAT_WORKSPACE_TOO_SMALL;
  if (((uintptr_t)d_ws & 255) || ((uintptr_t)d_hidden_k & 15) || ((uintptr_t)d_W & 15)) return NAT_INVALID_ARG;
  nat_status st = clear_diag(d_diag, (hipStream_t)stream);
  if (st != NAT_OK) return st;
  LogpArgs a{d_hidden_k, d_W, d_ids_k, N_k, H, V, d_logp_k, d_entropy_k, d_ws, ws_bytes, (hipStream_t)stream, d_diag};
  return dtype == NAT_DTYPE_BF16 ? logp_bf16_run(a) : logp_f32_run(a);
}

extern "C" nat_status nat_loss_fwd_bwd_kl(const void* d_hidden_k, const void* d_W, const int32_t* d_ids_k,
                                          const float* d_old_logp_k, const float* d_adv, const int32_t* d_kept_seq,
                                          const float* d_kept_w, int32_t N_k, int32_t H, int32_t V, int32_t dtype,
                                          float eps_lo, float eps_hi, float grad_scale,
                                          const float* d_ref_logp_k, float beta_kl, int32_t kl_kind,
                                          float* d_loss, float* d_logp_k, float* d_kl_k, float* d_entropy_k,
                                          int32_t* d_diag, void* d_dH_k, float* d_dW, int32_t accumulate_dw,
                                          void* d_ws, size_t ws_bytes, void* stream) {
  if (dtype != NAT_DTYPE_F32 && dtype != NAT_DTYPE_BF16) return NAT_UNSUPPORTED_DTYPE;
  if (N_k < 0 || !(eps_lo >= 0.f) || !(eps_hi >= 0.f) || !(beta_kl >= 0.f)) return NAT_INVALID_ARG;
  if (kl_kind != NAT_KL_LOG_RATIO && kl_kind != NAT_KL_NONNEG) return NAT_INVALID_ARG;
  if (H <= 0 || V <= 0) return NAT_BAD_SHAPE;
  if (dtype == NAT_DTYPE_BF16 && (H % 64) != 0) return NAT_BAD_SHAPE;
  if (!d_W || !d_loss || !d_dW) return NAT_INVALID_ARG;
  if (N_k > 0 && (!d_hidden_k || !d_ids_k || !d_old_logp_k || !d_adv || !d_kept_seq || !d_kept_w || !d_dH_k))
    return NAT_INVALID_ARG;
  if (N_k > 0 && beta_kl != 0.f && !d_ref_logp_k) return NAT_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  if (N_k == 0) {
    nat_status st = fill_zero_f32(d_loss, 1, s);
    if (st != NAT_OK) return st;
    st = clear_diag(d_diag, s);
    if (st != NAT_OK) return st;
    return accumulate_dw ? NAT_OK : fill_zero_f32(d_dW, (size_t)V * (size_t)H, s);
  }
  if (!d_ws || ws_bytes < nat_loss_workspace_min_bytes(N_k, H, V, dtype)) return NAT_WORKSPACE_TOO_SMALL;
  // the kernels use 16-byte accesses on the caller's arrays and 256-byte aligned workspace sections
  if (((uintptr_t)d_ws & 255) || ((uintptr_t)d_hidden_k & 15) || ((uintptr_t)d_W & 15) || ((uintptr_t)d_dH_k & 15) ||
      ((uintptr_t)d_dW & 15))
    return NAT_INVALID_ARG;
  nat_status st_diag = clear_diag(d_diag, s);
  if (st_diag != NAT_OK) return st_diag;
  LossArgs a{d_hidden_k, d_W, d_ids_k, d_old_logp_k, d_adv, d_kept_seq, d_kept_w, N_k, H, V,
             eps_lo, eps_hi, grad_scale, d_loss, d_logp_k, d_dH_k, d_dW, accumulate_dw, d_ws, ws_bytes, s,
             d_ref_logp_k, beta_kl, kl_kind, d_kl_k, d_entropy_k, d_diag};
  return dtype == NAT_DTYPE_BF16 ? loss_bf16_run(a) : loss_f32_run(a);
}

extern "C" nat_status nat_loss_fwd_bwd(const void* d_hidden_k, const void* d_W, const int32_t* d_ids_k,
                                       const float* d_old_logp_k, const float* d_adv, const int32_t* d_kept_seq,
                                       const float* d_kept_w, int32_t N_k, int32_t H, int32_t V, int32_t dtype,
                                       float eps_lo, float eps_hi, float grad_scale,
                                       float* d_loss, float* d_logp_k, void* d_dH_k, float* d_dW,
                                       int32_t accumulate_dw, void* d_ws, size_t ws_bytes, void* stream) {
  return nat_loss_fwd_bwd_kl(d_hidden_k, d_W, d_ids_k, d_old_logp_k, d_adv, d_kept_seq, d_kept_w, N_k, H, V, dtype,
                             eps_lo, eps_hi, grad_scale, nullptr, 0.f, NAT_KL_LOG_RATIO, d_loss, d_logp_k, nullptr,
                             nullptr, nullptr, d_dH_k, d_dW, accumulate_dw, d_ws, ws_bytes, stream);
}
