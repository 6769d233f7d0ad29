// bf16 path of nat_loss_fwd_bwd for gfx950: LM-head projection, full-vocabulary
// log-softmax, clipped GRPO surrogate with Horvitz-Thompson weights (Eq. 1, 3, 5,
// 6/9) and the gradients dH, dW (App. A) on the kept tokens.
//
// Tokens are processed in chunks of at most `cap` rows.  Per chunk:
//   logits GEMM   Z^T tile = W_tile . H_chunk^T on bf16 MFMA with fp32 accumulators;
//                 the epilogue never stores Z: per (token, 128-row vocabulary
//                 granule) it keeps the local max m and sum s of exp(z - m), the
//                 target logit, and stores E = exp(z - m) as bf16 (soft-max
//                 numerators, relative precision preserved);
//   token stats   merge (m, s) over granules -> log-sum-exp, log-prob, ratio,
//                 clipped surrogate, c_k = dLoss/dlogp_k;
//   rescale       dZ = -c_k exp(m - lse_k) E, one-hot term applied in fp32 before
//                 rounding; written in both orientations;
//   dH GEMM       dH_chunk = dZ . W           (contraction over the vocabulary);
//   dW GEMM       dW (+)= dZ^T . H_chunk      (contraction over the chunk's tokens,
//                 fp32, one owner per output tile, chunks in order: deterministic).
// All three contractions run through one "NT" kernel (both operands contiguous
// along the contraction axis); W^T and H_chunk^T copies make that possible.
#include "nat_internal.h"
#include "grpo_scalar.hip.h"

namespace nat {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kBM = 256, kBN = 256, kBK = 64;     // block tile; 4 wavefronts of 128 x 128
constexpr int kThreads = 256;
constexpr int kGranule = 128;                     // vocabulary rows per soft-max partial
constexpr int kTileBytes = kBM * kBK * 2;         // 32 KiB per operand per stage
constexpr int kMaxChunk = 16384;                  // token rows per chunk (recommended workspace)

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float x) {
  const __bf16 b = (__bf16)x;
  return __builtin_bit_cast(uint16_t, b);
}

// ---------------------------------------------------------------- transpose ----
// out[c][r] = in[r][c] for r < R, c < C; out has R_pad columns, the tail zero-filled.
__global__ void __launch_bounds__(256)
transpose_bf16_kernel(const uint16_t* __restrict__ in, int64_t ld_in, int R, int C,
                      uint16_t* __restrict__ out, int64_t ld_out, int R_pad) {
  __shared__ uint16_t tile[64][66];
  const int r0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int j = ty; j < 64; j += 4) {
    const int r = r0 + j, c = c0 + tx;
    tile[j][tx] = (r < R && c < C) ? in[(int64_t)r * ld_in + c] : (uint16_t)0;
  }
  __syncthreads();
  for (int j = ty; j < 64; j += 4) {
    const int c = c0 + j, r = r0 + tx;
    if (c < C && r < R_pad) out[(int64_t)c * ld_out + r] = tile[tx][j];
  }
}

// ------------------------------------------------------------------- GEMM ----
struct GemmArgs {
  const uint16_t* A; int64_t lda; int M;     // A [M, K] row-major (rows beyond M-1 are clamped)
  const uint16_t* B; int64_t ldb; int N;     // B [N, K] row-major
  int K;                                     // multiple of kBK
  int tiles_m, tiles_n;
};

// Block id -> output tile.  Blocks are dealt round-robin to the 8 XCDs, so ids
// congruent mod 8 share an L2: give each XCD a contiguous range of tiles, walked
// in groups of 8 tile-rows so that concurrently resident blocks reuse A and B tiles.
__device__ __forceinline__ void tile_of_block(const GemmArgs& g, int& tm, int& tn) {
  const int total = g.tiles_m * g.tiles_n;
  const int pid = blockIdx.x;
  int logical = pid;
  const int per_xcd = total / 8;
  if (pid < per_xcd * 8) logical = (pid & 7) * per_xcd + (pid >> 3);
  constexpr int kGroupM = 8;
  const int group_sz = kGroupM * g.tiles_n;
  const int group = logical / group_sz;
  const int first_m = group * kGroupM;
  const int rows = g.tiles_m - first_m < kGroupM ? g.tiles_m - first_m : kGroupM;
  const int in_group = logical - group * group_sz;
  tm = first_m + in_group % rows;
  tn = in_group / rows;
}

// 16-byte chunk c of row r of a [256][64] bf16 tile; XOR swizzle against bank conflicts.
__device__ __forceinline__ int lds_chunk_off(int r, int c) { return r * (kBK * 2) + ((c ^ (r & 7)) << 4); }

// Global -> LDS copy of one [256][64] bf16 operand tile without staging registers:
// each wavefront issues 8 direct-to-LDS loads of 16 bytes per lane.  One instruction
// fills 8 consecutive tile rows (1 KiB); the hardware places lane l at byte 16*l of
// that block, so the swizzle is applied by choosing which 16-byte chunk of the row
// each lane fetches: lane l -> row l/8, logical chunk (l%8) ^ (l/8).
struct TileLoader {
  const uint16_t* rowp[8];       // per-lane source pointer of each of the 8 loads (k = 0)

  __device__ __forceinline__ void init(const uint16_t* base, int64_t ld, int row0, int n_rows, int wave, int lane) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      int r = row0 + (j * 4 + wave) * 8 + (lane >> 3);
      r = r < n_rows ? r : n_rows - 1;
      rowp[j] = base + (int64_t)r * ld + (((lane & 7) ^ (lane >> 3)) << 3);
    }
  }
  __device__ __forceinline__ void issue(char* lds_tile, int k0, int wave) const {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(rowp[j] + k0),
          (__attribute__((address_space(3))) void*)(lds_tile + (j * 4 + wave) * 8 * (kBK * 2)), 16, 0, 0);
    }
  }
};

__device__ __forceinline__ void load_frags(const char* a_s, const char* b_s, int wm, int wn, int l32, int lhi, int ks,
                                           bf16x8 (&af)[4], bf16x8 (&bfr)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    af[i] = *(const bf16x8*)(a_s + lds_chunk_off(wm * 128 + i * 32 + l32, ks * 2 + lhi));
    bfr[i] = *(const bf16x8*)(b_s + lds_chunk_off(wn * 128 + i * 32 + l32, ks * 2 + lhi));
  }
}

// acc[mb][nb] element r of lane l is C[wm*128 + mb*32 + 8*(r/4) + 4*(l/32) + r%4][wn*128 + nb*32 + l%32]
template <class Epilogue>
__global__ void __launch_bounds__(kThreads, 1)
gemm_nt_kernel(GemmArgs g, Epilogue epi) {
  __shared__ __attribute__((aligned(1024))) char lds[2][2][kTileBytes];
  int tm, tn;
  tile_of_block(g, tm, tn);
  const int m0 = tm * kBM, n0 = tn * kBN;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, lhi = lane >> 5;

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  TileLoader la, lb;
  la.init(g.A, g.lda, m0, g.M, wave, lane);
  lb.init(g.B, g.ldb, n0, g.N, wave, lane);
  la.issue(lds[0][0], 0, wave);
  lb.issue(lds[0][1], 0, wave);
  __builtin_amdgcn_s_waitcnt(0x0f70);        // vmcnt(0): the direct-to-LDS loads have landed
  __syncthreads();

  const int kt_n = g.K / kBK;
  for (int kt = 0; kt < kt_n; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < kt_n) {
      la.issue(lds[cur ^ 1][0], (kt + 1) * kBK, wave);
      lb.issue(lds[cur ^ 1][1], (kt + 1) * kBK, wave);
    }
    const char* a_s = lds[cur][0];
    const char* b_s = lds[cur][1];
    bf16x8 af[2][4], bfr[2][4];
    load_frags(a_s, b_s, wm, wn, l32, lhi, 0, af[0], bfr[0]);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      if (ks < 3) load_frags(a_s, b_s, wm, wn, l32, lhi, ks + 1, af[(ks + 1) & 1], bfr[(ks + 1) & 1]);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks & 1][i], bfr[ks & 1][j], acc[i][j], 0, 0, 0);
    }
    __builtin_amdgcn_s_waitcnt(0x0f70);      // vmcnt(0)
    __syncthreads();
  }
  epi(acc, m0 + wm * 128, n0 + wn * 128, lane);
}

// ------------------------------------------------------------- epilogues ----

// Logits tile: rows = vocabulary (A = W), columns = tokens of the chunk (B = H_chunk).
struct LogitsEpilogue {
  int V, n_valid;                  // vocabulary size, valid tokens in the chunk
  int64_t ld_e;                    // leading dimension (tokens) of Et and of the partials
  uint16_t* Et;                    // [Vp, ld_e] bf16 out: exp(z - m_granule)
  float* m_part; float* s_part;    // [Vp/128, ld_e]
  float* z_target;                 // [ld_e]
  const int32_t* ids;              // target ids of the chunk's tokens

  __device__ __forceinline__ void operator()(f32x16 (&acc)[4][4], int v0, int k0, int lane) const {
    const int l32 = lane & 31, lhi = lane >> 5;
    const int granule = v0 / kGranule;
    const bool all_rows_valid = v0 + kGranule <= V;
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
      const int kk = k0 + nb * 32 + l32;                 // token column (always < ld_e)
      const int y = kk < n_valid ? ids[kk] : -1;
      float m = -INFINITY;
      if (all_rows_valid) {
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
          for (int r = 0; r < 16; ++r) m = fmaxf(m, acc[mb][nb][r]);
      } else {
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int v = v0 + mb * 32 + 8 * (r >> 2) + 4 * lhi + (r & 3);
            if (v >= V) acc[mb][nb][r] = -INFINITY;
            m = fmaxf(m, acc[mb][nb][r]);
          }
      }
      m = fmaxf(m, __shfl_xor(m, 32));
      // target logit, if the target row lies in this granule and in this lane's half
      const int yrel = y - v0;
      if (__any(yrel >= 0 && yrel < kGranule)) {
        if (yrel >= 0 && yrel < kGranule && ((yrel >> 2) & 1) == lhi) {
          float zt = 0.f;
#pragma unroll
          for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int r = 0; r < 16; ++r)
              if (yrel == mb * 32 + 8 * (r >> 2) + 4 * lhi + (r & 3)) zt = acc[mb][nb][r];
          z_target[kk] = zt;
        }
      }
      const float m_safe = m == -INFINITY ? 0.f : m;     // a granule entirely beyond V
      float s = 0.f;
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float e = __expf(acc[mb][nb][r] - m_safe);
          s += e;
          const int v = v0 + mb * 32 + 8 * (r >> 2) + 4 * lhi + (r & 3);
          Et[(int64_t)v * ld_e + kk] = f32_to_bf16_bits(e);
        }
      s += __shfl_xor(s, 32);
      if (lhi == 0) {
        m_part[(int64_t)granule * ld_e + kk] = m;
        s_part[(int64_t)granule * ld_e + kk] = s;
      }
    }
  }
};

// dH tile: rows = tokens of the chunk (A = dZ), columns = hidden units (B = W^T).
struct DHiddenEpilogue {
  int n_valid, H;
  uint16_t* dH;                    // rows of this chunk, [n_valid, H] bf16

  __device__ __forceinline__ void operator()(f32x16 (&acc)[4][4], int k0, int h0, int lane) const {
    const int l32 = lane & 31, lhi = lane >> 5;
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
      const int h = h0 + nb * 32 + l32;
      if (h >= H) continue;
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int k = k0 + mb * 32 + 8 * (r >> 2) + 4 * lhi + (r & 3);
          if (k < n_valid) dH[(int64_t)k * H + h] = f32_to_bf16_bits(acc[mb][nb][r]);
        }
    }
  }
};

// dW tile: rows = vocabulary (A = dZ^T), columns = hidden units (B = H_chunk^T).
struct DWeightEpilogue {
  int V, H, accumulate;
  float* dW;                       // [V, H] fp32

  __device__ __forceinline__ void operator()(f32x16 (&acc)[4][4], int v0, int h0, int lane) const {
    const int l32 = lane & 31, lhi = lane >> 5;
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
      const int h = h0 + nb * 32 + l32;
      if (h >= H) continue;
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int v = v0 + mb * 32 + 8 * (r >> 2) + 4 * lhi + (r & 3);
          if (v < V) {
            float* p = dW + (int64_t)v * H + h;
            *p = accumulate ? *p + acc[mb][nb][r] : acc[mb][nb][r];
          }
        }
    }
  }
};

// ------------------------------------------------- per-token statistics ----
__global__ void __launch_bounds__(256)
token_stats_kernel(const float* __restrict__ m_part, const float* __restrict__ s_part, int n_granules, int64_t ld,
                   const float* __restrict__ z_target, int n_valid, int chunk_start,
                   const float* __restrict__ old_logp, const float* __restrict__ adv,
                   const int32_t* __restrict__ kept_seq, const float* __restrict__ kept_w,
                   float eps_lo, float eps_hi, float grad_scale,
                   float* __restrict__ lse_out, float* __restrict__ c_out, float* __restrict__ logp_chunk,
                   float* __restrict__ logp_out, float* __restrict__ term) {
  const int kk = blockIdx.x * blockDim.x + threadIdx.x;
  if (kk >= n_valid) return;
  float m = -INFINITY;
  for (int gi = 0; gi < n_granules; ++gi) m = fmaxf(m, m_part[(int64_t)gi * ld + kk]);
  float s = 0.f;
  for (int gi = 0; gi < n_granules; ++gi) {
    const float mg = m_part[(int64_t)gi * ld + kk];
    if (mg != -INFINITY) s += s_part[(int64_t)gi * ld + kk] * __expf(mg - m);
  }
  const float lse = m + logf(s);
  const float logp = z_target[kk] - lse;
  const int k = chunk_start + kk;
  const float w = kept_w[k];
  const TokenScalars ts = grpo_token_scalars(logp, old_logp[k], adv[kept_seq[k]], w, eps_lo, eps_hi, grad_scale);
  lse_out[kk] = lse;
  c_out[kk] = ts.c;
  logp_chunk[kk] = logp;
  if (logp_out) logp_out[k] = logp;
  term[k] = w * ts.S;
}

// ------------------------------------------------------------- rescale ----
// Et [Vp, ld] holds E = exp(z - m_granule).  In place: dZ^T = -c_k exp(m_granule - lse_k) E
// with the target entry replaced by c_k (1 - softmax_target); also writes dZ [ld rows, Vp].
__global__ void __launch_bounds__(256)
rescale_kernel(uint16_t* __restrict__ Et, int64_t ld, uint16_t* __restrict__ dZ, int64_t ld_z,
               const float* __restrict__ m_part, const float* __restrict__ lse, const float* __restrict__ c,
               const float* __restrict__ logp_chunk, const int32_t* __restrict__ ids, int n_valid) {
  __shared__ uint16_t tile[64][66];
  const int v0 = blockIdx.x * 64, k0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int kk = k0 + tx;
  const bool valid = kk < n_valid;
  const int granule = v0 / kGranule;
  float alpha = 0.f, c_k = 0.f, onehot_val = 0.f;
  int y = -1;
  if (valid) {
    c_k = c[kk];
    const float mg = m_part[(int64_t)granule * ld + kk];
    alpha = mg == -INFINITY ? 0.f : -c_k * __expf(mg - lse[kk]);
    y = ids[kk];
    onehot_val = c_k * (1.f - __expf(logp_chunk[kk]));
  }
  for (int j = ty; j < 64; j += 4) {
    const int v = v0 + j;
    const int64_t off = (int64_t)v * ld + kk;
    const float e = __builtin_bit_cast(float, (uint32_t)Et[off] << 16);
    const float dz = (v == y) ? onehot_val : alpha * e;
    const uint16_t bits = valid ? f32_to_bf16_bits(dz) : (uint16_t)0;
    Et[off] = bits;
    tile[j][tx] = bits;
  }
  __syncthreads();
  for (int j = ty; j < 64; j += 4) {
    const int k = k0 + j;
    dZ[(int64_t)k * ld_z + v0 + tx] = tile[tx][j];
  }
}

// -------------------------------------------------------------- host side ----
static inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

struct Bf16Plan {
  int64_t Vp; int n_granules; int cap;          // padded vocabulary, granules, chunk capacity (tokens)
  size_t off_Wt, off_Et, off_dZ, off_Hkt, off_m, off_s, off_zt, off_lse, off_c, off_logp, off_term, total;
};

static Bf16Plan make_plan(int32_t N_k, int32_t H, int32_t V, int cap) {
  Bf16Plan p;
  p.Vp = round_up(V, kBM);
  p.n_granules = (int)(p.Vp / kGranule);
  p.cap = cap;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += (bytes + 255) / 256 * 256; return o; };
  p.off_Wt = take((size_t)H * p.Vp * 2);
  p.off_Et = take((size_t)p.Vp * cap * 2);
  p.off_dZ = take((size_t)cap * p.Vp * 2);
  p.off_Hkt = take((size_t)H * cap * 2);
  p.off_m = take((size_t)p.n_granules * cap * 4);
  p.off_s = take((size_t)p.n_granules * cap * 4);
  p.off_zt = take((size_t)cap * 4);
  p.off_lse = take((size_t)cap * 4);
  p.off_c = take((size_t)cap * 4);
  p.off_logp = take((size_t)cap * 4);
  p.off_term = take((size_t)(N_k > 0 ? N_k : 1) * 4);
  p.total = off;
  return p;
}

static int recommended_cap(int32_t N_k) {
  int64_t cap = round_up(N_k > 0 ? N_k : 1, kBN);
  return (int)(cap > kMaxChunk ? kMaxChunk : cap);
}

size_t loss_bf16_workspace_bytes(int32_t N_k, int32_t H, int32_t V, bool minimal) {
  return make_plan(N_k, H, V, minimal ? kBN : recommended_cap(N_k)).total;
}

template <class Epi>
static nat_status launch_gemm(const GemmArgs& g, const Epi& epi, int prof_class, hipStream_t s) {
  ProfScope prof(prof_class, s);
  gemm_nt_kernel<Epi><<<g.tiles_m * g.tiles_n, kThreads, 0, s>>>(g, epi);
  NAT_LAUNCH_CHECK();
  return NAT_OK;
}

nat_status loss_bf16_run(const LossArgs& a) {
  // largest chunk capacity (multiple of 256 tokens) whose plan fits the workspace
  int cap = recommended_cap(a.N_k);
  while (cap > kBN && make_plan(a.N_k, a.H, a.V, cap).total > a.ws_bytes) cap -= kBN;
  const Bf16Plan p = make_plan(a.N_k, a.H, a.V, cap);
  if (p.total > a.ws_bytes) return NAT_WORKSPACE_TOO_SMALL;
  hipStream_t s = a.stream;
  char* ws = (char*)a.ws;
  uint16_t* Wt = (uint16_t*)(ws + p.off_Wt);
  uint16_t* Et = (uint16_t*)(ws + p.off_Et);
  uint16_t* dZ = (uint16_t*)(ws + p.off_dZ);
  uint16_t* Hkt = (uint16_t*)(ws + p.off_Hkt);
  float* m_part = (float*)(ws + p.off_m);
  float* s_part = (float*)(ws + p.off_s);
  float* zt = (float*)(ws + p.off_zt);
  float* lse = (float*)(ws + p.off_lse);
  float* c = (float*)(ws + p.off_c);
  float* logp_chunk = (float*)(ws + p.off_logp);
  float* term = (float*)(ws + p.off_term);
  const uint16_t* W = (const uint16_t*)a.W;
  const uint16_t* hidden = (const uint16_t*)a.hidden;
  const int H = a.H, V = a.V;
  const int Vp = (int)p.Vp;
  const int tiles_h = (H + kBN - 1) / kBN;

  {  // W^T [H, Vp], vocabulary tail zero-filled
    ProfScope prof(PC_TRANSPOSE, s);
    transpose_bf16_kernel<<<dim3(Vp / 64, (H + 63) / 64), 256, 0, s>>>(W, H, V, H, Wt, Vp, Vp);
    NAT_LAUNCH_CHECK();
  }
  for (int c0 = 0; c0 < a.N_k; c0 += cap) {
    const int nv = a.N_k - c0 < cap ? a.N_k - c0 : cap;
    const int np = (int)round_up(nv, kBN);
    const uint16_t* hid_c = hidden + (int64_t)c0 * H;
    {  // H_chunk^T [H, np] (leading dimension cap), token tail zero-filled
      ProfScope prof(PC_TRANSPOSE, s);
      transpose_bf16_kernel<<<dim3(np / 64, (H + 63) / 64), 256, 0, s>>>(hid_c, H, nv, H, Hkt, cap, np);
      NAT_LAUNCH_CHECK();
    }
    {  // logits: rows = vocabulary, columns = tokens
      GemmArgs g{W, H, V, hid_c, H, nv, H, Vp / kBM, np / kBN};
      LogitsEpilogue e{V, nv, cap, Et, m_part, s_part, zt, a.ids + c0};
      nat_status st = launch_gemm(g, e, PC_LOGITS, s);
      if (st != NAT_OK) return st;
    }
    {
      ProfScope prof(PC_TOKEN_STATS, s);
      token_stats_kernel<<<(nv + 255) / 256, 256, 0, s>>>(m_part, s_part, p.n_granules, cap, zt, nv, c0, a.old_logp,
                                                         a.adv, a.kept_seq, a.kept_w, a.eps_lo, a.eps_hi,
                                                         a.grad_scale, lse, c, logp_chunk, a.logp, term);
      NAT_LAUNCH_CHECK();
    }
    {
      ProfScope prof(PC_RESCALE, s);
      rescale_kernel<<<dim3(Vp / 64, np / 64), 256, 0, s>>>(Et, cap, dZ, Vp, m_part, lse, c, logp_chunk,
                                                           a.ids + c0, nv);
      NAT_LAUNCH_CHECK();
    }
    {  // dH: rows = tokens, columns = hidden units, contraction over the padded vocabulary
      GemmArgs g{dZ, Vp, np, Wt, Vp, H, Vp, np / kBM, tiles_h};
      DHiddenEpilogue e{nv, H, (uint16_t*)a.dH + (int64_t)c0 * H};
      nat_status st = launch_gemm(g, e, PC_DHIDDEN, s);
      if (st != NAT_OK) return st;
    }
    {  // dW: rows = vocabulary, columns = hidden units, contraction over the chunk's tokens
      GemmArgs g{Et, cap, Vp, Hkt, cap, H, np, Vp / kBM, tiles_h};
      DWeightEpilogue e{V, H, (c0 > 0 || a.accumulate_dw) ? 1 : 0, a.dW};
      nat_status st = launch_gemm(g, e, PC_DWEIGHT, s);
      if (st != NAT_OK) return st;
    }
  }
  ProfScope prof(PC_LOSS_REDUCE, s);
  loss_reduce_kernel<<<1, 1024, 0, s>>>(term, a.N_k, a.loss);
  NAT_LAUNCH_CHECK();
  return NAT_OK;
}

}  // namespace nat
