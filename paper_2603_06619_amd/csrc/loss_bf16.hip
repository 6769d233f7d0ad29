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
// along the contraction axis).  Every operand is kept in a blocked layout in the
// workspace: blocks of 256 rows x 32 k-elements (16 KiB, contiguous), ordered k-fastest
// inside a 256-row tile, so a workgroup streams one contiguous region per operand
// instead of 256 strided rows.  W and H_chunk are repacked (plain and transposed);
// the soft-max numerators and dZ are produced directly in that layout.
#include "nat_internal.h"
#include "grpo_scalar.hip.h"

namespace nat {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kBM = 256, kBN = 256, kBK = 32;     // block tile; 4 wavefronts of 128 x 128
constexpr int kStages = 4;                        // LDS ring of k-slices (4 x 32 KiB)
constexpr int kThreads = 256;
constexpr int kGranule = 128;                     // vocabulary rows per soft-max partial
constexpr int kTileBytes = kBM * kBK * 2;         // 16 KiB per operand per stage
constexpr int kLoadsPerWave = 2 * (kTileBytes / 1024) / 4;   // direct-to-LDS loads per wavefront per stage (A and B)
constexpr int kMaxChunk = 32768;                  // token rows per chunk (recommended workspace)

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float x) {
  const __bf16 b = (__bf16)x;
  return __builtin_bit_cast(uint16_t, b);
}

// ------------------------------------------------------------ blocked layout ----
constexpr int kBlkElems = 256 * 32;               // one block: 256 rows x 32 k-elements

// element (row, k) of an operand with kb = K/32 k-slices
__host__ __device__ __forceinline__ int64_t blk_off(int row, int k, int kb) {
  return ((int64_t)(row >> 8) * kb + (k >> 5)) * kBlkElems + ((row & 255) << 5) + (k & 31);
}

// Repack a row-major matrix in [R, C] (leading dimension ld_in) into the blocked layout,
// in one or both orientations, zero-filling the padding:
//   out_rk: rows = r (padded to Rp, multiple of 256), k = c (C must be a multiple of 32);
//   out_cr: rows = c (padded to Cp, multiple of 256), k = r (padded to Rp).
__global__ void __launch_bounds__(256)
pack_blocked_kernel(const uint16_t* __restrict__ in, int64_t ld_in, int R, int C, int Rp, int Cp,
                    uint16_t* __restrict__ out_rk, uint16_t* __restrict__ out_cr) {
  __shared__ uint16_t tile[64][66];
  const int r0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int j = ty; j < 64; j += 4) {
    const int r = r0 + j, c = c0 + tx;
    const uint16_t x = (r < R && c < C) ? in[(int64_t)r * ld_in + c] : (uint16_t)0;
    tile[j][tx] = x;
    if (out_rk && c < C) out_rk[blk_off(r, c, C >> 5)] = x;
  }
  if (!out_cr) return;
  __syncthreads();
  for (int j = ty; j < 64; j += 4) {
    const int c = c0 + j, r = r0 + tx;
    out_cr[blk_off(c, r, Rp >> 5)] = tile[tx][j];
  }
}

// ------------------------------------------------------------------- GEMM ----
struct GemmArgs {
  const uint16_t* A;          // [tiles_m * 256, K] in the blocked layout
  const uint16_t* B;          // [tiles_n * 256, K] in the blocked layout
  int K;                      // multiple of kBK
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

// Byte offset of 16-byte chunk c (0..3) of row r in a [256][32] bf16 LDS tile (64-byte rows).
// A ds_read_b128 is served 16 lanes at a time over 64 banks; 16 consecutive rows at one
// chunk index would fall on 4 bank groups, so the chunk is XOR-ed with bits 2..3 of the row.
__device__ __forceinline__ int lds_chunk_off(int r, int c) { return r * (kBK * 2) + ((c ^ ((r >> 2) & 3)) << 4); }

// Global -> LDS copy of one [256][32] bf16 operand block (16 KiB, contiguous in memory)
// without staging registers: each wavefront issues 4 direct-to-LDS loads of 16 bytes per
// lane.  One instruction fills 16 consecutive tile rows (1 KiB); the hardware places lane l
// at byte 16*l of that KiB, so the LDS swizzle is applied by choosing which 16-byte chunk of
// its row a lane fetches: lane l -> row l/4, logical chunk (l%4) ^ ((l/16)%4).
struct TileLoader {
  static constexpr int kLoads = kTileBytes / 1024 / 4;      // per wavefront
  const uint16_t* src;           // this lane's chunk in k-slice 0 of load 0

  __device__ __forceinline__ void init(const uint16_t* base, int tile, int kb, int wave, int lane) {
    src = base + (int64_t)tile * kb * kBlkElems + (wave * 16 + (lane >> 2)) * kBK +
          (((lane & 3) ^ ((lane >> 4) & 3)) << 3);
  }
  __device__ __forceinline__ void issue(char* lds_tile, int kt, int wave) const {
    const uint16_t* p = src + (int64_t)kt * kBlkElems;
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(p + j * 64 * kBK),
          (__attribute__((address_space(3))) void*)(lds_tile + (j * 4 + wave) * 1024), 16, 0, 0);
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

// 8 of the 16 MFMAs of one k-substep: A fragments i0, i0+1 against all four B fragments
__device__ __forceinline__ void mfma_half(f32x16 (&acc)[4][4], const bf16x8 (&af)[4], const bf16x8 (&bfr)[4], int i0) {
#pragma unroll
  for (int i = i0; i < i0 + 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
}

// s_waitcnt immediates (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8)
constexpr int waitcnt_vm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0f70; }

// acc[mb][nb] element r of lane l is C[wm*128 + mb*32 + 8*(r/4) + 4*(l/32) + r%4][wn*128 + nb*32 + l%32]
template <class Epilogue>
__global__ void __launch_bounds__(kThreads, 1)
gemm_nt_kernel(GemmArgs g, Epilogue epi) {
  __shared__ __attribute__((aligned(1024))) char lds[kStages][2][kTileBytes];
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
  const int kt_n = g.K / kBK;
  la.init(g.A, tm, kt_n, wave, lane);
  lb.init(g.B, tn, kt_n, wave, lane);

  // Software pipeline over k-slices of 32.  Slice kt lives in lds[kt % 4]; three slices are
  // in flight while one is consumed, so a load has three iterations (96 MFMAs per wavefront)
  // to land.  Loads complete in issue order, hence "slice kt+1 has landed" is vmcnt(16): the
  // two younger slices (8 loads each per wavefront) may still be outstanding.  The barrier
  // sits before the second half of the slice's MFMAs, so the refill of the released buffer
  // and the first fragment reads of the next slice issue under those 16 MFMAs.  Slices past
  // the end re-load the last one (harmless) to keep the body branch-free and the count fixed.
#pragma unroll
  for (int st = 0; st < kStages; ++st) {
    const int k = st < kt_n ? st : kt_n - 1;
    la.issue(lds[st][0], k, wave);
    lb.issue(lds[st][1], k, wave);
  }
  __builtin_amdgcn_s_waitcnt(waitcnt_vm((kStages - 1) * kLoadsPerWave));
  __syncthreads();
  bf16x8 af[2][4], bfr[2][4];
  load_frags(lds[0][0], lds[0][1], wm, wn, l32, lhi, 0, af[0], bfr[0]);

  for (int kt = 0; kt < kt_n; ++kt) {
    const int cur = kt % kStages, nxt = (kt + 1) % kStages;
    // first k-substep of slice kt; the second substep's fragments are read under its first 8 MFMAs
    load_frags(lds[cur][0], lds[cur][1], wm, wn, l32, lhi, 1, af[1], bfr[1]);
    mfma_half(acc, af[0], bfr[0], 0);
    mfma_half(acc, af[0], bfr[0], 2);
#pragma unroll
    for (int x = 0; x < 8; ++x) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);     // 1 MFMA
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);     // 1 LDS read
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
    __builtin_amdgcn_sched_barrier(0);
    // slice kt+1 has landed (this wavefront's share; the barrier covers the others) and this
    // wavefront has finished reading slice kt, whose buffer is refilled below
    __builtin_amdgcn_s_waitcnt(waitcnt_vm((kStages - 2) * kLoadsPerWave) & 0xf0ff);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    // second k-substep; under it: first fragments of slice kt+1, then the refill of lds[cur]
    load_frags(lds[nxt][0], lds[nxt][1], wm, wn, l32, lhi, 0, af[0], bfr[0]);
    mfma_half(acc, af[1], bfr[1], 0);
    mfma_half(acc, af[1], bfr[1], 2);
    {
      int k2 = kt + kStages;
      k2 = k2 < kt_n ? k2 : kt_n - 1;
      la.issue(lds[cur][0], k2, wave);
      lb.issue(lds[cur][1], k2, wave);
    }
#pragma unroll
    for (int x = 0; x < 8; ++x) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);     // 1 MFMA
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);     // 1 LDS read
    }
#pragma unroll
    for (int x = 0; x < 8; ++x) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);     // 1 MFMA
      __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);     // 1 global->LDS load
    }
  }
  __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));   // no direct-to-LDS load may outlive the block
  __syncthreads();

  epi(acc, m0 + wm * 128, n0 + wn * 128, lane);
}

// ------------------------------------------------------------- epilogues ----

// Logits tile: rows = vocabulary (A = W), columns = tokens of the chunk (B = H_chunk).
struct LogitsEpilogue {
  int V, n_valid;                  // vocabulary size, valid tokens in the chunk
  int64_t ld_e;                    // leading dimension (tokens) of the partials
  int kb_e;                        // k-slices (padded tokens / 32) of Et
  uint16_t* Et;                    // blocked [Vp rows, padded tokens] bf16 out: exp(z - m_granule)
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
          Et[blk_off(v, kk, kb_e)] = f32_to_bf16_bits(e);
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
// 64 tokens per workgroup; the granules of a token are split over 4 wavefronts (granule
// gi goes to wavefront gi % 4), each keeping a running (max, sum); the four partial pairs
// are merged in wavefront order, so the result does not depend on timing.
__global__ void __launch_bounds__(256)
token_stats_kernel(const float* __restrict__ m_part, const float* __restrict__ s_part, int n_granules, int64_t ld,
                   const float* __restrict__ z_target, int n_valid, int chunk_start,
                   const float* __restrict__ old_logp, const float* __restrict__ adv,
                   const int32_t* __restrict__ kept_seq, const float* __restrict__ kept_w,
                   float eps_lo, float eps_hi, float grad_scale,
                   float* __restrict__ lse_out, float* __restrict__ c_out, float* __restrict__ logp_chunk,
                   float* __restrict__ logp_out, float* __restrict__ term) {
  __shared__ float m_s[4][64], s_s[4][64];
  const int t = threadIdx.x & 63, part = threadIdx.x >> 6;
  const int kk = blockIdx.x * 64 + t;
  float m = -INFINITY, s = 0.f;
  if (kk < n_valid) {
    for (int gi = part; gi < n_granules; gi += 4) {
      const float mg = m_part[(int64_t)gi * ld + kk];
      const float sg = s_part[(int64_t)gi * ld + kk];
      if (mg == -INFINITY) continue;                    // granule entirely beyond the vocabulary
      if (mg > m) { s = s * __expf(m - mg) + sg; m = mg; }
      else s += sg * __expf(mg - m);
    }
  }
  m_s[part][t] = m;
  s_s[part][t] = s;
  __syncthreads();
  if (part != 0 || kk >= n_valid) return;
  m = fmaxf(fmaxf(m_s[0][t], m_s[1][t]), fmaxf(m_s[2][t], m_s[3][t]));
  s = 0.f;
#pragma unroll
  for (int q = 0; q < 4; ++q)
    if (m_s[q][t] != -INFINITY) s += s_s[q][t] * __expf(m_s[q][t] - m);
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
// One block of Et (256 vocabulary rows x 32 tokens, 16 KiB contiguous) per workgroup.
// In place: dZ^T = -c_k exp(m_granule - lse_k) E, with the target entry replaced by
// c_k (1 - softmax_target) computed in fp32.  The same values are written transposed into
// dZ (rows = tokens, k = vocabulary), also blocked.
__global__ void __launch_bounds__(256)
rescale_kernel(uint16_t* __restrict__ Et, int kb_e, uint16_t* __restrict__ dZ, int kb_z,
               const float* __restrict__ m_part, int64_t ld_part, const float* __restrict__ lse,
               const float* __restrict__ c, const float* __restrict__ logp_chunk,
               const int32_t* __restrict__ ids, int n_valid) {
  __shared__ __attribute__((aligned(16))) uint16_t tr[32][256 + 8];   // [token][vocab row], padded rows
  __shared__ float alpha_s[2][32];
  __shared__ float onehot_s[32];
  __shared__ int y_s[32];
  const int vt = blockIdx.x, ks = blockIdx.y;          // vocabulary tile (256 rows), token slice (32)
  const int tid = threadIdx.x;
  if (tid < 64) {
    const int t = tid & 31, gsel = tid >> 5;
    const int kk = ks * 32 + t;
    float alpha = 0.f;
    if (kk < n_valid) {
      const float mg = m_part[(int64_t)(vt * 2 + gsel) * ld_part + kk];
      const float ck = c[kk];
      alpha = mg == -INFINITY ? 0.f : -ck * __expf(mg - lse[kk]);
      if (gsel == 0) {
        onehot_s[t] = ck * (1.f - __expf(logp_chunk[kk]));
        y_s[t] = ids[kk];
      }
    } else if (gsel == 0) {
      onehot_s[t] = 0.f;
      y_s[t] = -1;
    }
    alpha_s[gsel][t] = alpha;
  }
  __syncthreads();
  uint4* blk = (uint4*)(Et + ((int64_t)vt * kb_e + ks) * kBlkElems);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int q = i * 256 + tid;                       // 16-byte chunk: row q/4, tokens (q%4)*8 .. +7
    const int vr = q >> 2, t0 = (q & 3) << 3;
    const int v = vt * 256 + vr;
    const uint4 in = blk[q];
    const uint32_t w[4] = {in.x, in.y, in.z, in.w};
    uint32_t o[4];
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      uint32_t packed = 0;
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const int t = t0 + 2 * h + half;
        const float e = __builtin_bit_cast(float, (half ? (w[h] & 0xffff0000u) : (w[h] << 16)));
        const float dz = (v == y_s[t]) ? onehot_s[t] : alpha_s[vr >> 7][t] * e;
        const uint16_t bits = f32_to_bf16_bits(dz);
        tr[t][vr] = bits;
        packed |= (uint32_t)bits << (16 * half);
      }
      o[h] = packed;
    }
    blk[q] = make_uint4(o[0], o[1], o[2], o[3]);
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int q = i * 256 + tid;                       // token q/32, vocabulary rows (q%32)*8 .. +7
    const int t = q >> 5, vr0 = (q & 31) << 3;
    const int kk = ks * 32 + t;
    const uint4 val = *(const uint4*)&tr[t][vr0];
    *(uint4*)(dZ + blk_off(kk, vt * 256 + vr0, kb_z)) = val;
  }
}

// -------------------------------------------------------------- host side ----
static inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

struct Bf16Plan {
  int64_t Vp, Hp; int n_granules; int cap;      // padded vocabulary / hidden size, granules, chunk capacity (tokens)
  size_t off_Wb, off_Wtb, off_Hb, off_Hktb, off_Et, off_dZ, off_m, off_s, off_zt, off_lse, off_c, off_logp,
      off_term, total;
};

static Bf16Plan make_plan(int32_t N_k, int32_t H, int32_t V, int cap) {
  Bf16Plan p;
  p.Vp = round_up(V, kBM);
  p.Hp = round_up(H, kBN);
  p.n_granules = (int)(p.Vp / kGranule);
  p.cap = cap;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += (bytes + 255) / 256 * 256; return o; };
  p.off_Wb = take((size_t)p.Vp * H * 2);        // W:    rows = vocabulary, k = hidden
  p.off_Wtb = take((size_t)p.Hp * p.Vp * 2);    // W^T:  rows = hidden,     k = vocabulary
  p.off_Hb = take((size_t)cap * H * 2);         // H_chunk:   rows = tokens, k = hidden
  p.off_Hktb = take((size_t)p.Hp * cap * 2);    // H_chunk^T: rows = hidden, k = tokens
  p.off_Et = take((size_t)p.Vp * cap * 2);      // E then dZ^T: rows = vocabulary, k = tokens
  p.off_dZ = take((size_t)cap * p.Vp * 2);      // dZ:   rows = tokens, k = vocabulary
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
  uint16_t* Wb = (uint16_t*)(ws + p.off_Wb);
  uint16_t* Wtb = (uint16_t*)(ws + p.off_Wtb);
  uint16_t* Hb = (uint16_t*)(ws + p.off_Hb);
  uint16_t* Hktb = (uint16_t*)(ws + p.off_Hktb);
  uint16_t* Et = (uint16_t*)(ws + p.off_Et);
  uint16_t* dZ = (uint16_t*)(ws + p.off_dZ);
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
  const int Vp = (int)p.Vp, Hp = (int)p.Hp;

  {  // W and W^T in the blocked layout, padding zero-filled
    ProfScope prof(PC_TRANSPOSE, s);
    pack_blocked_kernel<<<dim3(Vp / 64, Hp / 64), 256, 0, s>>>(W, H, V, H, Vp, Hp, Wb, Wtb);
    NAT_LAUNCH_CHECK();
  }
  for (int c0 = 0; c0 < a.N_k; c0 += cap) {
    const int nv = a.N_k - c0 < cap ? a.N_k - c0 : cap;
    const int np = (int)round_up(nv, kBN);
    {  // H_chunk and H_chunk^T in the blocked layout
      ProfScope prof(PC_TRANSPOSE, s);
      pack_blocked_kernel<<<dim3(np / 64, Hp / 64), 256, 0, s>>>(hidden + (int64_t)c0 * H, H, nv, H, np, Hp, Hb, Hktb);
      NAT_LAUNCH_CHECK();
    }
    {  // logits: rows = vocabulary, columns = tokens, contraction over the hidden size
      GemmArgs g{Wb, Hb, H, Vp / kBM, np / kBN};
      LogitsEpilogue e{V, nv, cap, np / 32, Et, m_part, s_part, zt, a.ids + c0};
      nat_status st = launch_gemm(g, e, PC_LOGITS, s);
      if (st != NAT_OK) return st;
    }
    {
      ProfScope prof(PC_TOKEN_STATS, s);
      token_stats_kernel<<<(nv + 63) / 64, 256, 0, s>>>(m_part, s_part, p.n_granules, cap, zt, nv, c0, a.old_logp,
                                                         a.adv, a.kept_seq, a.kept_w, a.eps_lo, a.eps_hi,
                                                         a.grad_scale, lse, c, logp_chunk, a.logp, term);
      NAT_LAUNCH_CHECK();
    }
    {
      ProfScope prof(PC_RESCALE, s);
      rescale_kernel<<<dim3(Vp / 256, np / 32), 256, 0, s>>>(Et, np / 32, dZ, Vp / 32, m_part, cap, lse, c,
                                                            logp_chunk, a.ids + c0, nv);
      NAT_LAUNCH_CHECK();
    }
    {  // dH: rows = tokens, columns = hidden units, contraction over the padded vocabulary
      GemmArgs g{dZ, Wtb, Vp, np / kBM, Hp / kBN};
      DHiddenEpilogue e{nv, H, (uint16_t*)a.dH + (int64_t)c0 * H};
      nat_status st = launch_gemm(g, e, PC_DHIDDEN, s);
      if (st != NAT_OK) return st;
    }
    {  // dW: rows = vocabulary, columns = hidden units, contraction over the chunk's (padded) tokens
      GemmArgs g{Et, Hktb, np, Vp / kBM, Hp / kBN};
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
