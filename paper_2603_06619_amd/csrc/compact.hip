// nat_compact / nat_compact_pi: stable mask -> index compaction of the selected
// tokens with the Horvitz-Thompson weight of Eq. 6 / Eq. 9 folded with the
// 1/G * 1/|o_i| averaging of Eq. 5 (inclusion probability from the scheme's
// closed form, or read from a per-token array), plus an optional gather of the
// kept rows.
//
// Three passes over the bit mask: per-tile population counts, an exclusive scan
// of the tile counts, and a scatter in which each wavefront ranks its 64 tokens
// with a ballot prefix so that consecutive lanes write consecutive outputs.
#include "nat_internal.h"

#include <mutex>

namespace nat {

constexpr int kTileTokens = 4096;                 // tokens per scatter block
constexpr int kTileWords = kTileTokens / 32;      // 128 mask words
constexpr int kScatterThreads = 256;              // 4 wavefronts x 1024 tokens

__device__ __forceinline__ int wave_sum(int v) {
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

// tile_count[b] = number of kept tokens among packed positions [b*4096, (b+1)*4096)
__global__ void __launch_bounds__(kTileWords)
compact_count_kernel(const uint32_t* __restrict__ mask_bits, int64_t n_words, int32_t* __restrict__ tile_count) {
  __shared__ int part[kTileWords / 64];
  const int64_t w = (int64_t)blockIdx.x * kTileWords + threadIdx.x;
  const int c = wave_sum(w < n_words ? __popc(mask_bits[w]) : 0);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = c;
  __syncthreads();
  if (threadIdx.x == 0) tile_count[blockIdx.x] = part[0] + part[1];
}

// tile_offset[0..n_tiles] = exclusive scan of tile_count; n_kept = total.  One block.
__global__ void __launch_bounds__(1024)
compact_scan_kernel(const int32_t* __restrict__ tile_count, int n_tiles, int32_t* __restrict__ tile_offset,
                    int32_t* __restrict__ n_kept) {
  __shared__ int wave_tot[16];
  __shared__ int carry_s;
  if (threadIdx.x == 0) carry_s = 0;
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int base = 0; base < n_tiles; base += 1024) {
    const int j = base + threadIdx.x;
    const int v = j < n_tiles ? tile_count[j] : 0;
    int incl = v;                                   // inclusive scan inside the wavefront
    for (int off = 1; off < 64; off <<= 1) {
      const int up = __shfl_up(incl, off);
      if (lane >= off) incl += up;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    int before = carry_s;
    for (int w = 0; w < wave; ++w) before += wave_tot[w];
    if (j < n_tiles) tile_offset[j] = before + incl - v;
    __syncthreads();
    if (threadIdx.x == 1023) carry_s = before + incl;
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    tile_offset[n_tiles] = carry_s;
    *n_kept = carry_s;
  }
}

// Horvitz-Thompson weight of kept token t (1-based) of a rollout of length T.
__device__ __forceinline__ float ht_weight(int scheme, int64_t T, int64_t t, double n_rollouts, double p, int64_t C) {
  double w;
  if (scheme == NAT_SCHEME_URS) {
    w = 1.0 / (n_rollouts * (double)T * p);
  } else {
    int64_t Ci = C < 1 ? 1 : C;
    if (Ci > T) Ci = T;
    if (scheme == NAT_SCHEME_RPC && t > Ci) {
      w = (double)(T - Ci + 1) / ((double)(T - t + 1) * (double)T * n_rollouts);
    } else {
      w = 1.0 / (n_rollouts * (double)T);
    }
  }
  return (float)w;
}

__global__ void __launch_bounds__(kScatterThreads)
compact_scatter_kernel(SelectArgs a, double n_rollouts, const double* __restrict__ pi,
                       const uint32_t* __restrict__ mask_bits, int64_t n_words, int64_t n_tokens, int64_t kept_cap,
                       const int64_t* __restrict__ cu, int B, const int32_t* __restrict__ tile_offset,
                       int32_t* __restrict__ kept_idx, int32_t* __restrict__ kept_seq, float* __restrict__ kept_w) {
  __shared__ int wave_cnt[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // this wavefront's 1024 tokens = 32 mask words
  const int64_t word0 = (int64_t)blockIdx.x * kTileWords + wave * 32;
  const int64_t wi = word0 + lane;
  const uint32_t my_word = (lane < 32 && wi < n_words) ? mask_bits[wi] : 0u;
  const int cnt = wave_sum(__popc(my_word));
  if (lane == 0) wave_cnt[wave] = cnt;
  __syncthreads();
  int base = tile_offset[blockIdx.x];
  for (int w = 0; w < wave; ++w) base += wave_cnt[w];
  // rollouts touched by this wavefront's 1024 tokens: two wave-uniform searches bound the per-lane ones
  const int64_t N = cu[B];
  const int64_t span_first = word0 * 32;
  int i_lo = 0, i_hi = B;
  if (span_first < N) {
    const int64_t span_last = span_first + 1023 < N ? span_first + 1023 : N - 1;
    i_lo = rollout_of_pos(cu, 0, B, span_first);
    i_hi = rollout_of_pos(cu, i_lo, B, span_last) + 1;
  }

  for (int it = 0; it < 16; ++it) {
    const uint32_t lo = __shfl(my_word, 2 * it), hi = __shfl(my_word, 2 * it + 1);
    const uint64_t group = (uint64_t)lo | ((uint64_t)hi << 32);
    if (group == 0) continue;                                   // wave-uniform
    const bool keep = (group >> lane) & 1ull;
    const int rank = __popcll(group & ((1ull << lane) - 1ull));
    const int64_t n = (word0 + 2 * it) * 32 + lane;
    // entries beyond the outputs' capacity are counted but not written; a set bit at a position the
    // per-token arrays do not have (a foreign mask) is ranked but reads and writes nothing
    if (keep && base + rank < kept_cap && n < n_tokens) {
      const int i = rollout_of_pos(cu, i_lo, i_hi, n);
      const int64_t start = cu[i];
      const int64_t T = cu[i + 1] - start;
      const int scheme = a.scheme_per_rollout ? a.scheme_per_rollout[i] : a.scheme;
      const int out = base + rank;
      kept_idx[out] = (int32_t)n;
      kept_seq[out] = i;
      kept_w[out] = pi ? (float)(1.0 / ((n_rollouts * (double)T) * pi[n]))
                       : ht_weight(scheme, T, n - start + 1, n_rollouts, a.p, a.min_cut);
    }
    base += __popcll(group);
  }
}

// cu_kept[i] = number of kept tokens at packed positions < cu[i]
__global__ void compact_cu_kept_kernel(const uint32_t* __restrict__ mask_bits, const int64_t* __restrict__ cu, int B,
                                       int64_t n_tokens, const int32_t* __restrict__ tile_offset,
                                       int32_t* __restrict__ cu_kept) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i > B) return;
  const int64_t pos = cu[i] < 0 ? 0 : cu[i] > n_tokens ? n_tokens : cu[i];   // the mask holds n_tokens positions
  const int64_t tile = pos / kTileTokens;
  int c = tile_offset[tile];
  const int64_t w0 = tile * kTileWords, w1 = pos >> 5;
  for (int64_t w = w0; w < w1; ++w) c += __popc(mask_bits[w]);
  const int rem = (int)(pos & 31);
  if (rem) c += __popc(mask_bits[w1] & ((1u << rem) - 1u));
  cu_kept[i] = c;
}

// One block per kept row: copy row kept_idx[k] of `src` (row_bytes, multiple of 16) to row k.
__global__ void __launch_bounds__(256)
gather_rows_kernel(const int32_t* __restrict__ kept_idx, const int32_t* __restrict__ n_kept, int64_t rows_cap,
                   const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t row_vec16,
                   const int32_t* __restrict__ ids, int32_t* __restrict__ ids_k,
                   const float* __restrict__ old_logp, float* __restrict__ old_logp_k) {
  const int nk = *n_kept;
  for (int64_t k = blockIdx.x; k < nk && k < rows_cap; k += gridDim.x) {
    const int64_t n = kept_idx[k];
    if (src) {
      const uint4* s = src + n * row_vec16;
      uint4* d = dst + k * row_vec16;
      for (int64_t j = threadIdx.x; j < row_vec16; j += blockDim.x) d[j] = s[j];
    }
    if (threadIdx.x == 0) {
      if (ids) ids_k[k] = ids[n];
      if (old_logp) old_logp_k[k] = old_logp[n];
    }
  }
}

constexpr int64_t n_tiles_of(int64_t N) { return (N + kTileTokens - 1) / kTileTokens; }

// tile_count[n_tiles] + tile_offset[n_tiles + 1], int32, rounded up to 256 bytes
constexpr size_t compact_ws_bytes(int64_t N) {
  return (((size_t)(2 * n_tiles_of(N) + 1) * sizeof(int32_t) + 255) / 256) * 256 + 256;
}

// Scratch of nat_compact_static: the tile counts and offsets of up to NAT_COMPACT_STATIC_MAX_TOKENS
// tokens (about 513 KiB), resident on every GPU the library runs on until the process ends.  In host
// code this name stands for the symbol, not for a device address: the address on each device comes
// from hipGetSymbolAddress (static_scratch below) and only that pointer is handed to kernels.
constexpr size_t kStaticScratchBytes = compact_ws_bytes(NAT_COMPACT_STATIC_MAX_TOKENS);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices];          // per device: each GPU has its own copy at its own address

// Address of `scratch` on the current device, looked up once per device.
static nat_status static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return NAT_HIP_ERROR;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return NAT_HIP_ERROR;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return NAT_OK;
}

}  // namespace nat

using namespace nat;

extern "C" size_t nat_compact_workspace_bytes(int64_t N) {
  if (N < 0) return 0;
  return compact_ws_bytes(N);
}

namespace nat {

nat_status compact_run(const SelectArgs& a, const CompactArgs& c) {
  if (!c.cu || !c.cu_kept || !c.n_kept || c.B <= 0 || c.N < 0 || c.N >= (int64_t(1) << 31) ||
      c.n_rollouts_global <= 0 || c.kept_cap < 0)
    return NAT_INVALID_ARG;
  if (c.N > 0 && !c.mask_bits) return NAT_INVALID_ARG;
  if (c.N > 0 && c.kept_cap > 0 && (!c.kept_idx || !c.kept_seq || !c.kept_w)) return NAT_INVALID_ARG;
  if ((c.hidden != nullptr) != (c.hidden_k != nullptr) || (c.ids != nullptr) != (c.ids_k != nullptr) ||
      (c.old_logp != nullptr) != (c.old_logp_k != nullptr))
    return NAT_INVALID_ARG;
  int64_t row_bytes = 0;
  if (c.hidden) {
    if (c.dtype != NAT_DTYPE_F32 && c.dtype != NAT_DTYPE_BF16) return NAT_UNSUPPORTED_DTYPE;
    if (c.H <= 0) return NAT_BAD_SHAPE;
    row_bytes = (int64_t)c.H * (c.dtype == NAT_DTYPE_F32 ? 4 : 2);
    if (row_bytes % 16 != 0) return NAT_BAD_SHAPE;
    if (((uintptr_t)c.hidden & 15) || ((uintptr_t)c.hidden_k & 15)) return NAT_INVALID_ARG;   // 16-byte row copies
  }
  if (!c.ws || c.ws_bytes < nat_compact_workspace_bytes(c.N)) return NAT_WORKSPACE_TOO_SMALL;

  hipStream_t s = c.stream;
  const int64_t n_tiles = n_tiles_of(c.N);
  const int64_t n_words = nat_mask_words(c.N);
  int32_t* tile_count = (int32_t*)c.ws;
  int32_t* tile_offset = tile_count + n_tiles;
  {
    ProfScope prof(PC_COMPACT, s, !c.no_timing);
    if (n_tiles > 0) {
      compact_count_kernel<<<(unsigned)n_tiles, kTileWords, 0, s>>>(c.mask_bits, n_words, tile_count);
      NAT_LAUNCH_CHECK();
    }
    compact_scan_kernel<<<1, 1024, 0, s>>>(tile_count, (int)n_tiles, tile_offset, c.n_kept);
    NAT_LAUNCH_CHECK();
    if (n_tiles > 0) {
      compact_scatter_kernel<<<(unsigned)n_tiles, kScatterThreads, 0, s>>>(
          a, (double)c.n_rollouts_global, c.pi, c.mask_bits, n_words, c.N, c.kept_cap, c.cu, c.B, tile_offset,
          c.kept_idx, c.kept_seq, c.kept_w);
      NAT_LAUNCH_CHECK();
    }
    compact_cu_kept_kernel<<<(c.B + 1 + 255) / 256, 256, 0, s>>>(c.mask_bits, c.cu, c.B, c.N, tile_offset, c.cu_kept);
    NAT_LAUNCH_CHECK();
  }
  if (c.h_n_kept) NAT_HIP_TRY(hipMemcpyAsync(c.h_n_kept, c.n_kept, sizeof(int32_t), hipMemcpyDeviceToHost, s));
  const int64_t gather_rows = c.N < c.kept_cap ? c.N : c.kept_cap;
  if (gather_rows > 0 && (c.hidden || c.ids || c.old_logp)) {
    ProfScope prof(PC_GATHER, s, !c.no_timing);
    const int64_t grid = gather_rows < 65536 * 4 ? gather_rows : 65536 * 4;
    gather_rows_kernel<<<(unsigned)grid, 256, 0, s>>>(c.kept_idx, c.n_kept, gather_rows, (const uint4*)c.hidden,
                                                     (uint4*)c.hidden_k, row_bytes / 16, c.ids, c.ids_k,
                                                     c.old_logp, c.old_logp_k);
    NAT_LAUNCH_CHECK();
  }
  return NAT_OK;
}

}  // namespace nat

extern "C" nat_status nat_compact(const nat_select_params* params, int32_t n_rollouts_global,
                                  const uint32_t* d_mask_bits, const int64_t* d_cu_seqlens, int32_t B, int64_t N,
                                  int64_t kept_cap, int32_t* d_kept_idx, int32_t* d_kept_seq, float* d_kept_w, int32_t* d_cu_kept,
                                  int32_t* d_n_kept, int32_t* h_n_kept,
                                  const void* d_hidden, void* d_hidden_k, int32_t H, int32_t dtype,
                                  const int32_t* d_ids, int32_t* d_ids_k,
                                  const float* d_old_logp, float* d_old_logp_k,
                                  void* d_ws, size_t ws_bytes, void* stream) {
  SelectArgs a;
  nat_status st = validate_select(params, &a);
  if (st != NAT_OK) return st;
  return compact_run(a, CompactArgs{n_rollouts_global, d_mask_bits, nullptr, d_cu_seqlens, B, N, kept_cap, d_kept_idx,
                                    d_kept_seq, d_kept_w, d_cu_kept, d_n_kept, h_n_kept, d_hidden, d_hidden_k, H,
                                    dtype, d_ids, d_ids_k, d_old_logp, d_old_logp_k, d_ws, ws_bytes,
                                    (hipStream_t)stream, false});
}

extern "C" nat_status nat_compact_pi(int32_t n_rollouts_global, const uint32_t* d_mask_bits, const double* d_pi,
                                     const int64_t* d_cu_seqlens, int32_t B, int64_t N,
                                     int64_t kept_cap, int32_t* d_kept_idx, int32_t* d_kept_seq, float* d_kept_w, int32_t* d_cu_kept,
                                     int32_t* d_n_kept, int32_t* h_n_kept,
                                     const void* d_hidden, void* d_hidden_k, int32_t H, int32_t dtype,
                                     const int32_t* d_ids, int32_t* d_ids_k,
                                     const float* d_old_logp, float* d_old_logp_k,
                                     void* d_ws, size_t ws_bytes, void* stream) {
  if (N > 0 && !d_pi) return NAT_INVALID_ARG;
  SelectArgs a{};
  a.scheme = NAT_SCHEME_FULL;
  a.min_cut = 1;
  a.p = 1.0;
  return compact_run(a, CompactArgs{n_rollouts_global, d_mask_bits, d_pi, d_cu_seqlens, B, N, kept_cap, d_kept_idx,
                                    d_kept_seq, d_kept_w, d_cu_kept, d_n_kept, h_n_kept, d_hidden, d_hidden_k, H,
                                    dtype, d_ids, d_ids_k, d_old_logp, d_old_logp_k, d_ws, ws_bytes,
                                    (hipStream_t)stream, false});
}

extern "C" nat_status nat_compact_static(const nat_select_params* params, int32_t n_rollouts_global,
                                         const uint32_t* d_mask_bits, const int64_t* d_cu_seqlens, int32_t B,
                                         int64_t N, int64_t kept_cap, int32_t* d_kept_idx, int32_t* d_kept_seq,
                                         float* d_kept_w, int32_t* d_cu_kept, int32_t* d_n_kept, int32_t* h_n_kept,
                                         const void* d_hidden, void* d_hidden_k, int32_t H, int32_t dtype,
                                         const int32_t* d_ids, int32_t* d_ids_k,
                                         const float* d_old_logp, float* d_old_logp_k, void* stream) {
  SelectArgs a;
  nat_status st = validate_select(params, &a);
  if (st != NAT_OK) return st;
  if (N > NAT_COMPACT_STATIC_MAX_TOKENS) return NAT_BAD_SHAPE;      // beyond the resident scratch
  void* ws = nullptr;
  st = static_scratch(&ws);
  if (st != NAT_OK) return st;
  // every word of the scratch that the kernels read is written earlier in the same call (the tile
  // counts by the count pass, the offsets by the scan), so nothing has to be cleared between calls
  return compact_run(a, CompactArgs{n_rollouts_global, d_mask_bits, nullptr, d_cu_seqlens, B, N, kept_cap, d_kept_idx,
                                    d_kept_seq, d_kept_w, d_cu_kept, d_n_kept, h_n_kept, d_hidden, d_hidden_k, H,
                                    dtype, d_ids, d_ids_k, d_old_logp, d_old_logp_k, ws, kStaticScratchBytes,
                                    (hipStream_t)stream, true});
}
