// bf16 path of nat_loss_fwd_bwd / nat_loss_fwd_bwd_kl / nat_logp_fwd for gfx950: LM-head
// projection, full-vocabulary log-softmax, clipped GRPO surrogate with Horvitz-Thompson
// weights (Eq. 1, 3, 5, 6/9), optional KL term (Eq. 4) and entropy, and the gradients dH, dW
// (App. A) on the kept tokens.  The forward pass alone runs the first two steps below and
// keeps only the sums.
//
// Tokens are processed in chunks of at most `cap` rows (16384 or 32768 with the recommended workspace); the
// forward sweep and the dH contraction of a chunk run in sub-chunks of 8192 rows.  Per chunk:
//   reference     ref_k = h_k . W[ids_k]: the target logit, used only as the exponent shift;
//   logits GEMM   Z^T tile = W_tile . H^T on bf16 MFMA with fp32 accumulators; the epilogue never
//                 stores Z: it stores E = exp(z - ref_k) as bf16, ONCE, rows = token (soft-max
//                 numerators: bf16 keeps their relative precision), per (token, 128-row vocabulary
//                 granule) partial sums of E, and the exact target logit;
//   token stats   S_k = sum of the partials (fixed order), lse = ref + log S, log-prob, ratio,
//                 clipped surrogate, c_k = dLoss/dlogp_k, beta_k = -c_k / S_k;
//                 dz_kv = beta_k E_kv, except the target entry c_k (1 - p_target), which is
//                 patched into E as -S_k (1 - p_target), computed in fp32 before rounding;
//   dH GEMM       dH = diag(beta) (E . W)            (contraction over the vocabulary);
//   dW GEMM       dW (+)= E^T . (diag(beta) H_chunk) (contraction over the chunk's tokens, fp32,
//                 one owner per output tile, chunks in order: deterministic).  Its A operand is
//                 the same copy of E, which is stored along this contraction's k axis: the tile
//                 is gathered in 2 KiB pieces and fragments are formed by the transposing LDS
//                 read (ds_read_b64_tr_b16).
// The shift by the target logit needs log(p_max / p_target) < 70 for every kept token (E is
// clamped there; the token statistics count the tokens this may have touched); a token the current
// policy gives less than e^-70 of its mode's probability does not occur for rollouts drawn from a
// behaviour policy inside the clip range.
// All three contractions run through one "NT" kernel (both operands contiguous along the
// contraction axis; the k-major A operand of dW is the one exception described above).  Every
// operand is kept in a blocked layout in the workspace: blocks of 256 rows x 32 k-elements (16 KiB,
// contiguous), ordered k-fastest inside a 256-row tile, so a workgroup streams one contiguous
// region per operand instead of 256 strided rows.  W and H_chunk are repacked (plain and
// transposed); the soft-max numerators are produced directly in that layout.
#include "nat_internal.h"
#include "grpo_scalar.hip.h"

#include <type_traits>

namespace nat {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));
// The soft-max numerators are written once and read back only by the two backward contractions,
// long after they have left the L2: non-temporal stores (1 % on the logits kernel).
#define NAT_E_STORE(ptr, val) __builtin_nontemporal_store((val), (ptr))

constexpr int kBM = 256, kBN = 256, kBK = 32;     // block tile: 4 wavefronts of 128 x 128 or 8 of 128 x 64
constexpr int kStages = 4;                        // LDS ring of k-slices (4 x 32 KiB)
constexpr int kGranule = 128;                     // vocabulary rows per soft-max partial
constexpr int kTileBytes = kBM * kBK * 2;         // 16 KiB per operand per stage
// Wavefronts per workgroup of each contraction (4: one per SIMD, 128 x 128 each, 256 accumulator
// registers; 8: two per SIMD, 128 x 64 each: row-major operands only).  Measured on the Qwen3-8B
// head with the row-major kernel: dH 2 % slower with 8, the logits contraction unchanged; the k-major
// dW loop is written for 4.
// Tile rows per group of the block -> tile map, per contraction (measured: 4 is 1-2 % faster than 8
// for the two backward contractions, 2 and 6 are slower, 16 is 8 % slower).
#ifndef NAT_GROUP_LOGITS
#define NAT_GROUP_LOGITS 8
#endif
#ifndef NAT_GROUP_DHIDDEN
#define NAT_GROUP_DHIDDEN 4
#endif
#ifndef NAT_GROUP_DWEIGHT
#define NAT_GROUP_DWEIGHT 4
#endif
#ifndef NAT_WAVES_LOGITS
#define NAT_WAVES_LOGITS 4
#endif
#ifndef NAT_WAVES_DHIDDEN
#define NAT_WAVES_DHIDDEN 4
#endif
#ifndef NAT_WAVES_DWEIGHT
#define NAT_WAVES_DWEIGHT 4
#endif
constexpr int kMaxChunk = 32768;                  // most token rows per chunk (see recommended_cap)
constexpr int kNumCU = 256;                       // compute units (one workgroup of these kernels each)
constexpr int kMinSlicesPerRange = 32;            // shortest range of a cut dW contraction axis (k-slices)
#ifndef NAT_SUBCHUNK
#define NAT_SUBCHUNK 8192
#endif
constexpr int kSubChunk = NAT_SUBCHUNK;           // smallest token count per launch of the logits and dH contractions

// two floats -> two bf16 in one 32-bit word (lo in bits 0..15): one packed conversion instruction
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float x) {
  const __bf16 b = (__bf16)x;
  return __builtin_bit_cast(uint16_t, b);
}

// ------------------------------------------------------------ blocked layout ----
constexpr int kBlkElems = 256 * 32;               // one block: 256 rows x 32 k-elements

// element (row, k) of an operand with kb = K/32 k-slices.  Inside a row of a block the four
// 16-byte chunks are stored permuted (chunk index XOR bits 2..3 of the row): a block is then a
// byte-for-byte image of the bank-conflict-free LDS tile, and the direct-to-LDS copy reads it
// linearly, 16 bytes per lane.
__host__ __device__ __forceinline__ int64_t blk_off(int row, int k, int kb) {
  return ((int64_t)(row >> 8) * kb + (k >> 5)) * kBlkElems + ((row & 255) << 5) +
         (((((k & 31) >> 3) ^ ((row >> 2) & 3))) << 3) + (k & 7);
}

// Repack a row-major matrix in [R, C] (leading dimension ld_in) into the blocked layout,
// in one or both orientations, zero-filling the padding:
//   out_rk: rows = r (padded to Rp, multiple of 256), k = c (C must be a multiple of 32);
//   out_cr: rows = c (padded to Cp, multiple of 256), k = r (padded to Rp).
//   row_scale: optional [R] factor applied to row r of the input in out_cr (fp32 product, rounded once).
//   kb_cr: k-slices of the operand out_cr belongs to (Rp / 32 when the input is the whole operand;
//          more when the rows are a range of a longer contraction axis: out_cr then points at the
//          range's first k-slice).
// One workgroup repacks a 64 x 64 tile, 16 bytes (8 elements) per access on the global side: rows of
// the input and 16-byte chunks of the blocked layout are both 16-byte aligned (C and ld_in multiples
// of 8, pointers 16-byte aligned: checked at the entry points).
__global__ void __launch_bounds__(256)
pack_blocked_kernel(const uint16_t* __restrict__ in, int64_t ld_in, int R, int C, int Rp, int Cp,
                    uint16_t* __restrict__ out_rk, uint16_t* __restrict__ out_cr, int kb_cr,
                    const float* __restrict__ row_scale) {
  union Chunk { uint4 q; uint16_t e[8]; };
  __shared__ __attribute__((aligned(16))) uint16_t tile[64][72];     // 144-byte rows: 16-byte aligned chunks
  const int r0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
  const int cc = threadIdx.x & 7, jr = threadIdx.x >> 3;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int j = jr + 32 * i;
    const int r = r0 + j, c = c0 + 8 * cc;
    Chunk x;
    x.q = make_uint4(0u, 0u, 0u, 0u);
    if (r < R && c < C) x.q = *reinterpret_cast<const uint4*>(in + (int64_t)r * ld_in + c);
    if (out_rk && c < C) *reinterpret_cast<uint4*>(out_rk + blk_off(r, c, C >> 5)) = x.q;
    if (row_scale && r < R) {
      const float f = row_scale[r];
#pragma unroll
      for (int e = 0; e < 8; ++e) x.e[e] = f32_to_bf16_bits(__builtin_bit_cast(float, (uint32_t)x.e[e] << 16) * f);
    }
    *reinterpret_cast<uint4*>(&tile[j][8 * cc]) = x.q;
  }
  if (!out_cr) return;
  __syncthreads();
  // transposed: row c of the output holds k = r; the tile's 64 r are two k-slices, each a contiguous
  // 4 KiB (64 rows x 64 bytes) of the blocked operand; four neighbouring threads write one 64-byte row
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int q = threadIdx.x + 256 * i;
    const int cj = (q >> 2) & 63, rbase = (q >> 8) * 32 + (q & 3) * 8;
    Chunk y;
#pragma unroll
    for (int e = 0; e < 8; ++e) y.e[e] = tile[rbase + e][cj];
    *reinterpret_cast<uint4*>(out_cr + blk_off(c0 + cj, r0 + rbase, kb_cr)) = y.q;
  }
}

// ------------------------------------------------------------------- GEMM ----
struct GemmArgs {
  const uint16_t* A;          // [tiles_m * 256, K] in the blocked layout
  const uint16_t* B;          // [tiles_n * 256, K] in the blocked layout
  int K;                      // multiple of kBK
  int tiles_m, tiles_n;
  int group_m;                // tile rows walked together (see tile_of_block)
  int kb_a_src;               // k-major A only (see TileLoaderKMajor): k-slices of the source operand
  int k_splits;               // > 1: the contraction axis is cut into this many ranges of kt_per_split k-slices, one
  int kt_per_split;           // workgroup per (tile, range); the epilogue is told which slab its raw sums go to
  int tail_tiles;             // with k_splits > 1: 0 = every tile is cut (slab = range); T > 0 = only the last T tiles in
                              // launch order are (slab = position among them * k_splits + range), the others run whole
};

// Block id -> output tile.  Blocks are dealt round-robin to the 8 XCDs, so ids
// congruent mod 8 share an L2: give each XCD a contiguous range of tiles, walked
// in groups of `group_m` tile-rows so that concurrently resident blocks reuse A and B tiles.
__device__ __forceinline__ void tile_of_block(const GemmArgs& g, int pid, int& tm, int& tn) {
  const int total = g.tiles_m * g.tiles_n;
  int logical = pid;
  const int per_xcd = total / 8;
  if (pid < per_xcd * 8) logical = (pid & 7) * per_xcd + (pid >> 3);
  const int kGroupM = g.group_m;
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
// without staging registers: the NW wavefronts issue 16 direct-to-LDS loads of 16 bytes per
// lane between them.  One instruction copies 1 KiB (16 tile rows) linearly: the hardware
// places lane l at byte 16*l of that KiB, and the block in memory already has the LDS tile's
// chunk order.
template <int NW>
struct TileLoader {
  static constexpr int kLoads = kTileBytes / 1024 / NW;     // per wavefront
  const uint16_t* src;           // this lane's chunk in k-slice 0 of load 0

  // A wavefront copies kLoads consecutive KiB of the block (16 * kLoads rows): the loads of one
  // slice differ only in the instruction's immediate offset, which the hardware adds to both the
  // global and the LDS address, so one address and one LDS base serve all of them.
  __device__ __forceinline__ void init(const uint16_t* base, int tile, int kb, int wave, int lane) {
    src = base + (int64_t)tile * kb * kBlkElems + wave * (kLoads * 16 * kBK) + lane * 8;
  }
  __device__ __forceinline__ void start_at(int kt0) { src += (int64_t)kt0 * kBlkElems; }   // slice 0 := slice kt0
  // load kIdx = 0 .. kLoads - 1 of this wavefront's share
  template <int kIdx>
  __device__ __forceinline__ void issue_one(char* lds_tile, int kt, int wave) const {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + (int64_t)kt * kBlkElems),
                                     (__attribute__((address_space(3))) void*)(lds_tile + wave * (kLoads * 1024)), 16,
                                     kIdx * 1024, 0);
  }
  __device__ __forceinline__ void issue(char* lds_tile, int kt, int wave) const {
    const uint16_t* p = src + (int64_t)kt * kBlkElems;
    char* dst = lds_tile + wave * (kLoads * 1024);
    static_assert(kLoads == 4 || kLoads == 2, "immediate offsets below are written out");
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)p,
                                     (__attribute__((address_space(3))) void*)dst, 16, 0, 0);
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)p,
                                     (__attribute__((address_space(3))) void*)dst, 16, 1024, 0);
    if (kLoads == 4) {
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)p,
                                       (__attribute__((address_space(3))) void*)dst, 16, 2048, 0);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)p,
                                       (__attribute__((address_space(3))) void*)dst, 16, 3072, 0);
    }
  }
};

// The same copy for an A operand that is only stored with its rows along THIS contraction's k axis
// (the soft-max numerators: rows = token, k = vocabulary, read by the dW contraction whose k axis is
// the token).  A [256 rows][32 k] tile of the contraction is then eight pieces of the source, one per
// 32-row block of the tile: rows (kt % 8) * 32 .. + 31 of the source block (token tile kt / 8, k-slice
// 8 * tile + piece), 2 KiB contiguous each.  The LDS tile holds the pieces one after another, i.e.
// [row block][k][row within block], and fragments come out of it through the transposing LDS read.
template <int NW>
struct TileLoaderKMajor {
  static constexpr int kLoads = kTileBytes / 1024 / NW;     // per wavefront (4 with 4 wavefronts)
  static constexpr int kPieces = kLoads / 2;                // 2 KiB pieces per wavefront
  const uint16_t* src;           // this lane's 16 bytes of the wavefront's first piece, token tile 0, rows 0..15
  int64_t tile_stride;           // elements between consecutive token tiles of the source

  __device__ __forceinline__ void init(const uint16_t* base, int tile, int kb_src, int wave, int lane) {
    src = base + (int64_t)(8 * tile + wave * kPieces) * kBlkElems + lane * 8;
    tile_stride = (int64_t)kb_src * kBlkElems;
  }
  __device__ __forceinline__ void start_at(int kt0) { src += (int64_t)(kt0 >> 3) * tile_stride; }   // kt0 % 8 == 0
  // load kIdx = 0 .. kLoads - 1 of this wavefront's share (1 KiB: half a piece)
  template <int kIdx>
  __device__ __forceinline__ void issue_one(char* lds_tile, int kt, int wave) const {
    constexpr int piece = kIdx >> 1;
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void*)(src + (int64_t)(kt >> 3) * tile_stride + (kt & 7) * 1024 + (int64_t)piece * kBlkElems),
        (__attribute__((address_space(3))) void*)(lds_tile + (wave * kPieces + piece) * 2048), 16, (kIdx & 1) * 1024, 0);
  }
};

// Per-lane byte offsets, inside a [k = 32][32 rows] piece, of the two transposing reads (q = 0, 1)
// that make one A fragment of k-substep 0.  The transposing read works on groups of 16 lanes: lane
// i of a group supplies the address of 4 consecutive 16-bit elements and receives element i % 4 of
// the lanes i / 4, i / 4 + 4, i / 4 + 8, i / 4 + 12.  With lane i pointing at k = K0 + i / 4 and rows
// 16 g + 4 (i % 4) .. + 3, lane i ends up with row 16 g + i and k = K0 .. K0 + 3: the MFMA's A layout
// (row = lane % 32, 8 consecutive k from 8 * (lane / 32)) after two reads, K0 = 8 * (lane / 32) + 4 q.
// The 16-byte chunks of a source row are stored XOR-ed with bits 2..3 of the row (see blk_off); for
// these k values that is 2 * (lane / 32) + q.  The 32 lanes of a half-wavefront then cover all 64
// LDS banks exactly once.
struct KMajorFragOffsets {
  int off[2];
  __device__ __forceinline__ void init(int lane) {
    const int i = lane & 15, g = (lane >> 4) & 1, lhi = lane >> 5, a = i & 3;
#pragma unroll
    for (int q = 0; q < 2; ++q)
      off[q] = (8 * lhi + 4 * q + (i >> 2)) * 64 + ((((2 * g + (a >> 1)) ^ (2 * lhi + q)) & 3) << 4) + (a & 1) * 8;
  }
};

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

// One k-substep of the row-major loop, instruction slot by slot (the compiler may not move anything
// across a slot's end): slot m holds MFMA m on the fragments (au, bu); behind each of the first 4 + NB
// MFMAs one fragment read of k-substep ks_load from (a_s, b_s) into (al, bl); the remaining MFMAs carry
// the direct-to-LDS loads of this wavefront's share of slice k into lds_dst, evenly spaced (mixing them
// with the fragment reads measured slower).
template <int NW, int NB, int M = 0>
__device__ __forceinline__ void substep_slots(f32x16 (&acc)[4][NB], const bf16x8 (&au)[4], const bf16x8 (&bu)[NB],
                                              bf16x8 (&al)[4], bf16x8 (&bl)[NB], const char* a_s, const char* b_s,
                                              int a_row0, int b_row0, int l32, int lhi, int ks_load,
                                              const TileLoader<NW>& ld, char* lds_dst, int k, int wave) {
  constexpr int kLoadFirst = 4 + NB, kLoadEvery = (4 * NB - kLoadFirst) / TileLoader<NW>::kLoads;
  static_assert(kLoadEvery >= 1, "every load needs a slot");
  if constexpr (M < 4 * NB) {
    constexpr int i = M / NB, j = M % NB;
    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(au[i], bu[j], acc[i][j], 0, 0, 0);
    if constexpr (M < 4) al[M] = *(const bf16x8*)(a_s + lds_chunk_off(a_row0 + M * 32 + l32, ks_load * 2 + lhi));
    else if constexpr (M < 4 + NB) bl[M - 4] = *(const bf16x8*)(b_s + lds_chunk_off(b_row0 + (M - 4) * 32 + l32, ks_load * 2 + lhi));
    if constexpr (M >= kLoadFirst && (M - kLoadFirst) % kLoadEvery == 0 && (M - kLoadFirst) / kLoadEvery < TileLoader<NW>::kLoads)
      ld.template issue_one<(M - kLoadFirst) / kLoadEvery>(lds_dst, k, wave);
    __builtin_amdgcn_sched_barrier(0);
    substep_slots<NW, NB, M + 1>(acc, au, bu, al, bl, a_s, b_s, a_row0, b_row0, l32, lhi, ks_load, ld, lds_dst, k, wave);
  }
}

__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)p;
}

// The transposing read as inline assembly (byte offset as an immediate): invisible to the compiler's wait-count
// pass, which would otherwise put a wait for all direct-to-LDS loads in front of it; the caller waits
// (lgkmcnt) before it uses what was read.
__device__ __forceinline__ s16x4 lds_read_tr16_b64(uint32_t addr, int off) {
  s16x4 v;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "i"(off) : "memory");
  return v;
}

// One k-substep of the k-major loop with 4 wavefronts of 128 x 128, slot by slot (see substep_slots): MFMA m on
// (au, bu); behind the first 8 MFMAs one transposing read each (halves q = m % 2 of A block m / 2, from the
// piece bases a_rd[q]) and behind the first 4 also one 16-byte read of B; behind MFMAs 8, 10, 12, 14 one
// direct-to-LDS load of the refill (the A tile's when kRefillA, else the B tile's).
template <bool kRefillA, int M = 0>
__device__ __forceinline__ void substep_slots_kmajor4(f32x16 (&acc)[4][4], const bf16x8 (&au)[4], const bf16x8 (&bu)[4],
                                                      s16x4 (&al)[8], bf16x8 (&bl)[4], const uint32_t (&a_rd)[2], const char* b_rd,
                                                      const TileLoaderKMajor<4>& la, const TileLoader<4>& lb, char* lds_dst,
                                                      int k, int wave) {
  if constexpr (M < 16) {
    constexpr int i = M / 4, j = M % 4;
    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(au[i], bu[j], acc[i][j], 0, 0, 0);
    if constexpr (M < 4) bl[M] = *(const bf16x8*)(b_rd + M * 2048);
    if constexpr (M < 8) al[M] = lds_read_tr16_b64(a_rd[M & 1], (M / 2) * 2048);
    if constexpr (M >= 8 && (M & 1) == 0) {
      if constexpr (kRefillA) la.template issue_one<(M - 8) / 2>(lds_dst, k, wave);
      else lb.template issue_one<(M - 8) / 2>(lds_dst, k, wave);
    }
    __builtin_amdgcn_sched_barrier(0);
    substep_slots_kmajor4<kRefillA, M + 1>(acc, au, bu, al, bl, a_rd, b_rd, la, lb, lds_dst, k, wave);
  }
}

// fragments of k-substep ks: four 32-row blocks of A from row a_row0, NB 32-row blocks of B from b_row0
template <int NB>
__device__ __forceinline__ void load_frags(const char* a_s, const char* b_s, int a_row0, int b_row0, int l32, int lhi,
                                           int ks, bf16x8 (&af)[4], bf16x8 (&bfr)[NB]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) af[i] = *(const bf16x8*)(a_s + lds_chunk_off(a_row0 + i * 32 + l32, ks * 2 + lhi));
#pragma unroll
  for (int j = 0; j < NB; ++j) bfr[j] = *(const bf16x8*)(b_s + lds_chunk_off(b_row0 + j * 32 + l32, ks * 2 + lhi));
}

// s_waitcnt immediates (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8)
constexpr int waitcnt_vm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0f70; }

// NW wavefronts in a 2 x (NW/2) grid over the 256 x 256 tile: wavefront (wm, wn) owns rows
// wm*128.. and columns wn*(NB*32).. with NB = 16/NW (4 wavefronts: 128 columns, 8: 64 columns).
// acc[mb][nb] element r of lane l is C[row0 + mb*32 + 8*(r/4) + 4*(l/32) + r%4][col0 + nb*32 + l%32]
// AT: the A operand is read from a source stored along this contraction's k axis (TileLoaderKMajor);
// g.kb_a_src is then the number of k-slices of that source.
template <class Epilogue, int NW, bool AT = false>
__global__ void __launch_bounds__(NW * 64, 1)
gemm_nt_kernel(GemmArgs g, Epilogue epi) {
  constexpr int NB = 16 / NW;                                  // 32-column blocks per wavefront
  constexpr int kLoadsPerWave = 2 * (kTileBytes / 1024) / NW;  // direct-to-LDS loads per wavefront per slice
  // one LDS object (with a second one the compiler's wait-count pass orders every fragment read behind all
  // direct-to-LDS loads in flight): the ring, and behind it the words the epilogue parks across the k-loop
  constexpr int kStashWords = Epilogue::template stash_words<16 / NW>();
  struct Shared {
    char ring[kStages][2][kTileBytes];
    int stash[kStashWords > 0 ? kStashWords * NW * 64 : 1];
  };
  __shared__ __attribute__((aligned(1024))) Shared sm;
  auto& lds = sm.ring;
  int* pre_stash = sm.stash;
  int tm, tn;
  const int n_tiles = g.tiles_m * g.tiles_n;
  int pid = (int)blockIdx.x, range = -1, slab = -1;           // range of the contraction axis / slab (-1: whole axis)
  if (g.k_splits > 1) {
    if (g.tail_tiles == 0) {
      range = pid / n_tiles;
      pid -= range * n_tiles;
      slab = range;
    } else if (pid >= n_tiles - g.tail_tiles) {
      const int r = pid - (n_tiles - g.tail_tiles);
      range = r / g.tail_tiles;
      const int pos = r - range * g.tail_tiles;
      pid = n_tiles - g.tail_tiles + pos;
      slab = pos * g.k_splits + range;
    }
  }
  tile_of_block(g, pid, tm, tn);
  const int m0 = tm * kBM, n0 = tn * kBN;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / (NW / 2), wn = wave % (NW / 2);
  const int a_row0 = wm * 128, b_row0 = wn * (NB * 32);
  const int l32 = lane & 31, lhi = lane >> 5;

  f32x16 acc[4][NB];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // per-column scalars the epilogue needs (token id, exponent shift): fetched into LDS now, read after the k-loop
  typename Epilogue::template Pre<NB> pre;
  epi.template prefetch<NB>(pre_stash, NW * 64, n0 + b_row0, lane, wave);

  typename std::conditional<AT, TileLoaderKMajor<NW>, TileLoader<NW>>::type la;
  TileLoader<NW> lb;
  const int kt_all = g.K / kBK;
  la.init(g.A, tm, AT ? g.kb_a_src : kt_all, wave, lane);
  lb.init(g.B, tn, kt_all, wave, lane);
  int kt_n = kt_all;                                           // k-slices this workgroup contracts over
  if (range >= 0) {
    const int kt0 = range * g.kt_per_split;                    // a multiple of 8 (TileLoaderKMajor::start_at)
    kt_n = kt_all - kt0 < g.kt_per_split ? kt_all - kt0 : g.kt_per_split;
    la.start_at(kt0);
    lb.start_at(kt0);
  }

  if constexpr (AT) {
    // k-major A: the row-major pipeline below (refill in two halves), with 4 wavefronts of 128 x 128, every
    // instruction of the loop placed by hand (substep_slots_kmajor4), and the A fragments through the transposing
    // read issued as inline assembly.  (The compiler's builtin for that read carries no memory operand, so its
    // wait-count pass puts a wait for ALL direct-to-LDS loads in flight in front of every such read: vmcnt(0)
    // inside the k-loop, 20-30 % slower.  As inline assembly the read is invisible to that pass; the kernel
    // waits for it itself, lgkmcnt(0) before the next substep uses what was read.  An earlier variant kept the
    // builtin read and hid the loads instead, with 8 wavefronts and compiler-scheduled reads: 3.5 % slower.)
    static_assert(NW == 4, "the k-major loop is written for 4 wavefronts");
    constexpr int kHalfLoads = kLoadsPerWave / 2;
    KMajorFragOffsets fo;
    fo.init(lane);
    const int a_blk0 = a_row0 / 32;
#pragma unroll
    for (int st = 0; st < kStages; ++st) {
      const int k = st < kt_n ? st : kt_n - 1;
      la.template issue_one<0>(lds[st][0], k, wave);
      la.template issue_one<1>(lds[st][0], k, wave);
      la.template issue_one<2>(lds[st][0], k, wave);
      la.template issue_one<3>(lds[st][0], k, wave);
      if (st < kStages - 1) lb.issue(lds[st][1], k, wave);
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_vm((2 * kStages - 3) * kHalfLoads));   // slice 0 has landed
    __syncthreads();
    s16x4 ah[2][8];
    bf16x8 bfr[2][4];
    auto a_bases = [&](int stage, int ks, uint32_t (&out)[2]) {
      const uint32_t piece0 = lds_addr(lds[stage][0] + a_blk0 * 2048 + ks * 1024);
      out[0] = piece0 + fo.off[0];
      out[1] = piece0 + fo.off[1];
    };
    auto join = [&](const s16x4 (&h)[8], bf16x8 (&out)[4]) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const s16x8 both = {h[2 * i][0], h[2 * i][1], h[2 * i][2], h[2 * i][3], h[2 * i + 1][0], h[2 * i + 1][1], h[2 * i + 1][2], h[2 * i + 1][3]};
        out[i] = __builtin_bit_cast(bf16x8, both);
      }
    };
    {
      uint32_t ar[2];
      a_bases(0, 0, ar);
#pragma unroll
      for (int m = 0; m < 8; ++m) ah[0][m] = lds_read_tr16_b64(ar[m & 1], (m / 2) * 2048);
#pragma unroll
      for (int j = 0; j < 4; ++j) bfr[0][j] = *(const bf16x8*)(lds[0][1] + lds_chunk_off(b_row0 + j * 32 + l32, lhi));
    }
    for (int kt = 0; kt < kt_n; ++kt) {
      const int cur = kt % kStages, nxt = (kt + 1) % kStages, last = (kt + kStages - 1) % kStages;
      int k1 = kt + kStages - 1;
      k1 = k1 < kt_n ? k1 : kt_n - 1;
      int k2 = kt + kStages;
      k2 = k2 < kt_n ? k2 : kt_n - 1;
      uint32_t ar[2];
      bf16x8 au[4];
      // first k-substep of slice kt: reads its second substep's fragments, refills the B tile of slice kt + 3
      a_bases(cur, 1, ar);
      __builtin_amdgcn_s_waitcnt(0xc07f);                      // lgkmcnt(0): the fragments read under the last substep
      join(ah[0], au);
      __builtin_amdgcn_sched_barrier(0);
      substep_slots_kmajor4<false>(acc, au, bfr[0], ah[1], bfr[1], ar, lds[cur][1] + lds_chunk_off(b_row0 + l32, 2 + lhi),
                                   la, lb, lds[last][1], k1, wave);
      __builtin_amdgcn_s_waitcnt(waitcnt_vm((kStages - 2) * kLoadsPerWave) & 0xf0ff);
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
      // second k-substep: reads the first fragments of slice kt + 1, refills the A tile of lds[cur] with slice kt + 4
      a_bases(nxt, 0, ar);
      join(ah[1], au);
      __builtin_amdgcn_sched_barrier(0);
      substep_slots_kmajor4<true>(acc, au, bfr[1], ah[0], bfr[0], ar, lds[nxt][1] + lds_chunk_off(b_row0 + l32, lhi),
                                  la, lb, lds[cur][0], k2, wave);
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));   // no direct-to-LDS load may outlive the block
    __syncthreads();
    epi(acc, pre, m0 + a_row0, n0 + b_row0, lane, wave, &lds[0][0][0], slab);
    return;
  } else {
  // Software pipeline over k-slices of 32.  Slice kt lives in lds[kt % 4]; three slices are
  // in flight while one is consumed, so a load has two to three iterations to land.  The barrier
  // sits between the two k-substeps of a slice; once it is passed, every wavefront has finished
  // reading slice kt and its buffer may be refilled.  The refill is issued in two halves so that
  // the loads of the NW wavefronts (which run in step) do not reach the CU's one address unit
  // all within a few hundred cycles: the A tile under the second substep of slice kt, the B tile
  // under the first substep of slice kt+1, each load one or two MFMAs after the previous one.
  // Loads complete in issue order (A0 B0 A1 B1 ...), hence "slice kt+1 has landed" at the barrier of
  // slice kt is vmcnt(2 * kLoadsPerWave): the halves of the two younger slices may be outstanding.
  // Slices past the end re-load the last one (into a buffer nobody reads again) to keep the body
  // branch-free and the count fixed.
  constexpr int kHalfLoads = kLoadsPerWave / 2;                // loads per wavefront and operand tile
#pragma unroll
  for (int st = 0; st < kStages; ++st) {
    const int k = st < kt_n ? st : kt_n - 1;
    la.issue(lds[st][0], k, wave);
    if (st < kStages - 1) lb.issue(lds[st][1], k, wave);
  }
  __builtin_amdgcn_s_waitcnt(waitcnt_vm((2 * kStages - 3) * kHalfLoads));   // slice 0 has landed
  __syncthreads();
  bf16x8 af[2][4], bfr[2][NB];
  load_frags<NB>(lds[0][0], lds[0][1], a_row0, b_row0, l32, lhi, 0, af[0], bfr[0]);

  for (int kt = 0; kt < kt_n; ++kt) {
    const int cur = kt % kStages, nxt = (kt + 1) % kStages, last = (kt + kStages - 1) % kStages;
    // first k-substep of slice kt; under its MFMAs: the second substep's fragments and the B half of
    // the refill of the buffer released at the previous barrier (slice kt + 3)
    int k1 = kt + kStages - 1;
    k1 = k1 < kt_n ? k1 : kt_n - 1;
    __builtin_amdgcn_sched_barrier(0);
    substep_slots<NW, NB>(acc, af[0], bfr[0], af[1], bfr[1], lds[cur][0], lds[cur][1], a_row0, b_row0, l32, lhi, 1,
                          lb, lds[last][1], k1, wave);
    // slice kt+1 has landed (this wavefront's share; the barrier covers the others) and this
    // wavefront has finished reading slice kt, whose buffer is refilled from here on
    __builtin_amdgcn_s_waitcnt(waitcnt_vm((kStages - 2) * kLoadsPerWave) & 0xf0ff);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    // second k-substep; under it: first fragments of slice kt+1 and the A half of the refill of lds[cur]
    int k2 = kt + kStages;
    k2 = k2 < kt_n ? k2 : kt_n - 1;
    substep_slots<NW, NB>(acc, af[1], bfr[1], af[0], bfr[0], lds[nxt][0], lds[nxt][1], a_row0, b_row0, l32, lhi, 0,
                          la, lds[cur][0], k2, wave);
  }
  __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));   // no direct-to-LDS load may outlive the block
  __syncthreads();

  epi.unstash(pre, pre_stash, NW * 64);
  epi(acc, pre, m0 + a_row0, n0 + b_row0, lane, wave, &lds[0][0][0], slab);
  }
}

// ------------------------------------------------------------- epilogues ----

// Logits tile: rows = vocabulary (A = W), columns = tokens of the chunk (B = H_chunk).
template <bool kEntropy, bool kStoreE = true>
struct LogitsEpilogue {
  int V, n_valid;                  // vocabulary size, valid tokens in the chunk
  int64_t ld_part;                 // leading dimension (tokens) of the partial sums
  int kb_z;                        // k-slices of Eb (Vp / 32)
  uint16_t* Eb;                    // blocked, rows = token, k = vocabulary: E = exp(z - ref), stored once
  float* s_part;                   // [Vp/128, ld_part] partial sums of E
  float* t_part;                   // [Vp/128, ld_part] partial sums of E (z - ref) (entropy), kEntropy only
  float* z_target;                 // [ld_part] exact target logits
  const int32_t* ids;              // target ids of the chunk's tokens
  const float* ref;                // [ld_part] exponent shift per token

  static constexpr int kStageRow = 272;        // bytes per token row of the LDS staging tile (128 bf16 + pad)

  // The per-column scalars the epilogue needs (token id, exponent shift) are fetched before the k-loop
  // straight into LDS (direct-to-LDS loads of 4 bytes per lane, from a clamped index; n_valid >= 1 in
  // every launch) and read back after it: they wait for nothing, hold no registers across the loop, and
  // are older than every operand load, so the loop's load counting is unchanged.  (Fetched into registers
  // they either cost a wait before the first operand loads, or live across the loop, where the compiler
  // spilled some of them and each reload in the epilogue waited for the stores in flight.)
  template <int NB> struct Pre { int y[NB]; float shift[NB]; };
  template <int NB> static constexpr int stash_words() { return 2 * NB; }
  template <int NB>
  __device__ __forceinline__ void prefetch(int* words, int n_threads, int k0, int lane, int wave) const {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int kk = k0 + nb * 32 + (lane & 31);
      const int kc = kk < n_valid ? kk : n_valid - 1;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(ids + kc),
                                       (__attribute__((address_space(3))) void*)(words + (2 * nb) * n_threads + wave * 64), 4, 0, 0);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(ref + kc),
                                       (__attribute__((address_space(3))) void*)(words + (2 * nb + 1) * n_threads + wave * 64), 4, 0, 0);
    }
  }
  template <int NB>
  __device__ __forceinline__ void unstash(Pre<NB>& pre, const int* words, int n_threads) const {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      pre.y[nb] = words[(2 * nb) * n_threads + threadIdx.x];
      pre.shift[nb] = __builtin_bit_cast(float, words[(2 * nb + 1) * n_threads + threadIdx.x]);
    }
  }

  template <int NB>
  __device__ __forceinline__ void operator()(f32x16 (&acc)[4][NB], const Pre<NB>& pre, int v0, int k0, int lane, int wave,
                                             char* lds, int) const {
    constexpr int kTok = NB * 32;                          // token columns of this wavefront
    const int l32 = lane & 31, lhi = lane >> 5;
    const int granule = v0 / kGranule;
    const bool all_rows_valid = v0 + kGranule <= V;
    constexpr float kLog2e = 1.44269504088896340736f, kLn2 = 0.69314718055994530942f;

    int y_of[NB];                  // target id of this lane's token per column block; -1: padding column, or
    float shift_of[NB];            // an id outside the vocabulary (matches no row)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const bool tok_valid = k0 + nb * 32 + l32 < n_valid;
      y_of[nb] = (tok_valid && pre.y[nb] >= 0 && pre.y[nb] < V) ? pre.y[nb] : -1;
      shift_of[nb] = tok_valid ? pre.shift[nb] : 0.f;
    }

    // exact target logit, if the target row lies in this granule and in this lane's half
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int yrel = y_of[nb] - v0;
      if (__any(yrel >= 0 && yrel < kGranule)) {
        if (yrel >= 0 && yrel < kGranule && ((yrel >> 2) & 1) == lhi) {
          float zt = 0.f;
#pragma unroll
          for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int r = 0; r < 16; ++r)
              if (yrel == mb * 32 + 8 * (r >> 2) + 4 * lhi + (r & 3)) zt = acc[mb][nb][r];
          z_target[k0 + nb * 32 + l32] = zt;
        }
      }
    }

    // One pass over the accumulators, 32 token columns (all 128 vocabulary rows of the wavefront) at a
    // time: E = exp(min(z - shift, 70)) as 2^(min(z * log2(e) - shift * log2(e), 70 * log2(e))) (one fma,
    // one min and the hardware exponential per logit, sixteen at a time with independent temporaries),
    // its running sums, and at once the store of those columns, so that the stores of one group are in
    // flight under the exponentials of the next.  E is stored once, rows = token, k = vocabulary (the
    // dH contraction reads it as it is, the dW contraction through the transposing LDS read): a lane
    // holds 4 consecutive vocabulary entries of its token; the 32 x 128 group is staged through this
    // wavefront's own part of the LDS ring (free after the k-loop) and leaves as 16-byte stores, 1 KiB
    // (16 token rows of one 32-wide vocabulary slice) contiguous per instruction.  The staging area is
    // private to the wavefront and LDS operations of one wavefront execute in order, so no barrier is
    // needed between its writes, its reads and the next group's writes.
    char* stage = lds + wave * (32 * kStageRow);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const float nshift2 = -shift_of[nb] * kLog2e;
      float s2[2] = {0.f, 0.f}, t2[2] = {0.f, 0.f};        // two independent chains per sum
#pragma unroll
      for (int mb = 0; mb < 4; ++mb) {
        float x2[16], e[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) x2[r] = fminf(fmaf(acc[mb][nb][r], kLog2e, nshift2), 70.f * kLog2e);
#pragma unroll
        for (int r = 0; r < 16; ++r) e[r] = __builtin_amdgcn_exp2f(x2[r]);
        if (!all_rows_valid) {                             // only the last vocabulary tile pays for the row check
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (v0 + mb * 32 + 8 * (r >> 2) + 4 * lhi + (r & 3) >= V) e[r] = 0.f;
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          s2[r & 1] += e[r];
          if (kEntropy) t2[r & 1] = fmaf(e[r], x2[r], t2[r & 1]);
        }
        if (kStoreE) {
#pragma unroll
          for (int r4 = 0; r4 < 4; ++r4) {
            uint2 w;
            w.x = pack_bf16x2(e[4 * r4], e[4 * r4 + 1]);
            w.y = pack_bf16x2(e[4 * r4 + 2], e[4 * r4 + 3]);
            *(uint2*)(stage + l32 * kStageRow + (mb * 32 + 8 * r4 + 4 * lhi) * 2) = w;
          }
        }
      }
      if (kStoreE) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {                      // vocabulary slice i / 2, token rows (i % 2) * 16 .. + 15
          const int sl = i >> 1, tok = (i & 1) * 16 + (lane >> 2), ch = lane & 3;
          const uint4 val = *(const uint4*)(stage + tok * kStageRow + sl * 64 + ch * 16);
          NAT_E_STORE((u32x4v*)(Eb + blk_off(k0 + nb * 32 + tok, v0 + sl * 32 + ch * 8, kb_z)), __builtin_bit_cast(u32x4v, val));
        }
      }
      const int kk = k0 + nb * 32 + l32;                   // token column (always inside the padded chunk)
      float sum = s2[0] + s2[1];
      sum += __shfl_xor(sum, 32);
      if (lhi == 0) s_part[(int64_t)granule * ld_part + kk] = sum;
      if (kEntropy) {
        float t = (t2[0] + t2[1]) * kLn2;                  // back to natural-log units
        t += __shfl_xor(t, 32);
        if (lhi == 0) t_part[(int64_t)granule * ld_part + kk] = t;
      }
    }
  }
};

// dH tile: rows = tokens of the chunk (A = E), columns = hidden units (B = W^T); rows scaled by beta.
struct DHiddenEpilogue {
  int n_valid, H;
  uint16_t* dH;                    // rows of this chunk, [n_valid, H] bf16
  const float* beta;               // [n_valid]
  float* partial;                  // split contraction: [k_splits][rows_p][cols_p] fp32 partial sums (else NULL)
  int rows_p, cols_p;              // padded token rows / hidden columns of the launch

  template <int NB> struct Pre {};
  template <int NB> static constexpr int stash_words() { return 0; }
  template <int NB> __device__ __forceinline__ void prefetch(int*, int, int, int, int) const {}
  template <int NB> __device__ __forceinline__ void unstash(Pre<NB>&, const int*, int) const {}
  template <int NB>
  __device__ __forceinline__ void operator()(f32x16 (&acc)[4][NB], const Pre<NB>&, int k0, int h0, int lane, int wave,
                                             char* lds, int slab_id) const {
    const int l32 = lane & 31, lhi = lane >> 5;
    if (slab_id >= 0) {            // this workgroup's range of the vocabulary: the raw sums go to its slab
      float* slab = partial + (int64_t)slab_id * rows_p * cols_p;
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int k = k0 + mb * 32 + 8 * (r >> 2) + 4 * lhi + (r & 3);
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) slab[(int64_t)k * cols_p + h0 + nb * 32 + l32] = acc[mb][nb][r];
        }
      return;
    }
    // 32 token rows at a time: beta_k * acc rounded to bf16 goes through this wavefront's own part of the LDS
    // ring (free after the k-loop; rows of NB * 64 + 16 bytes) and leaves as 16-byte stores, whole rows of the
    // wavefront's NB * 32 columns contiguous (2-byte stores straight from the accumulators took 80 k cycles
    // per tile).  LDS operations of one wavefront execute in order: no barrier between its writes and reads.
    constexpr int kRowBytes = NB * 64, kStageRow = kRowBytes + 16;
    constexpr int kChunks = kRowBytes / 16, kRowsPerStore = 64 / kChunks;
    char* stage = lds + wave * (32 * kStageRow);
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = 8 * (r >> 2) + 4 * lhi + (r & 3);
        const int k = k0 + mb * 32 + row;
        const float b = k < n_valid ? beta[k] : 0.f;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
          *(uint16_t*)(stage + row * kStageRow + (nb * 32 + l32) * 2) = f32_to_bf16_bits(b * acc[mb][nb][r]);
      }
#pragma unroll
      for (int i = 0; i < 32 / kRowsPerStore; ++i) {
        const int row = i * kRowsPerStore + lane / kChunks, ch = lane % kChunks;
        const uint4 val = *(const uint4*)(stage + row * kStageRow + ch * 16);
        const int k = k0 + mb * 32 + row, h = h0 + ch * 8;
        if (k < n_valid && h < H) *(uint4*)(dH + (int64_t)k * H + h) = val;     // H is a multiple of 8: whole chunks
      }
    }
  }
};

// dW tile: rows = vocabulary (A = E^T), columns = hidden units (B = (diag(beta) H_chunk)^T).
struct DWeightEpilogue {
  int V, H, accumulate;
  float* dW;                       // [V, H] fp32
  float* partial;                  // tiles whose contraction is cut into ranges: [slab][256][256] fp32 raw sums

  template <int NB> struct Pre {};
  template <int NB> static constexpr int stash_words() { return 0; }
  template <int NB> __device__ __forceinline__ void prefetch(int*, int, int, int, int) const {}
  template <int NB> __device__ __forceinline__ void unstash(Pre<NB>&, const int*, int) const {}
  // the wavefront's tile is MA x NB blocks of 32 x 32
  template <int MA, int NB, class P>
  __device__ __forceinline__ void operator()(f32x16 (&acc)[MA][NB], const P&, int v0, int h0, int lane, int,
                                             char*, int slab_id) const {
    const int l32 = lane & 31, lhi = lane >> 5;
    if (slab_id >= 0) {            // one range of this tile's tokens: raw sums to the slab, added up by dw_tail_reduce_kernel
      float* slab = partial + (int64_t)slab_id * (kBM * kBN);
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int mb = 0; mb < MA; ++mb)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            slab[((v0 & (kBM - 1)) + mb * 32 + 8 * (r >> 2) + 4 * lhi + (r & 3)) * kBN + (h0 & (kBN - 1)) + nb * 32 + l32] = acc[mb][nb][r];
      return;
    }
    // One owner per element and launch, launches in stream order: the atomic sum is that of a
    // read-modify-write, but the addition happens at the L2 and the workgroup does not wait for it.
    // Addresses are a wave-uniform row pointer plus one per-lane offset (rows 4 * lhi further down, column
    // l32), and the two launch-wide conditions (accumulate or overwrite, every row inside the vocabulary or
    // the last tile's row check) are taken once, outside the loops: per element that leaves the store or
    // atomic and a scalar add (per-element branches and 64-bit vector address arithmetic made this epilogue
    // 31 k cycles per tile).
    const uint32_t lane_off = (uint32_t)(4 * lhi) * (uint32_t)H + (uint32_t)l32;   // elements
    const bool rows_ok = v0 + MA * 32 <= V;
    auto sweep = [&](auto acc_mode, auto checked) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        if (h0 + nb * 32 >= H) continue;                     // H is a multiple of 64: a 32-column block is in or out
#pragma unroll
        for (int mb = 0; mb < MA; ++mb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int v = v0 + mb * 32 + 8 * (r >> 2) + (r & 3);   // row of lanes 0..31 (wave-uniform)
            if (decltype(checked)::value && v + 4 * lhi >= V) continue;
            float* p = dW + (int64_t)v * H + (h0 + nb * 32) + lane_off;
            if (decltype(acc_mode)::value) unsafeAtomicAdd(p, acc[mb][nb][r]);
            else *p = acc[mb][nb][r];
          }
      }
    };
    if (accumulate) {
      if (rows_ok) sweep(std::true_type{}, std::false_type{});
      else sweep(std::true_type{}, std::true_type{});
    } else {
      if (rows_ok) sweep(std::false_type{}, std::false_type{});
      else sweep(std::false_type{}, std::true_type{});
    }
  }
};

// dH of a launch whose contraction was split: dH[k][h] = beta_k * (slab 0 + slab 1 + ...), in slab order.
__global__ void __launch_bounds__(256)
dh_reduce_kernel(const float* __restrict__ partial, int k_splits, int rows_p, int cols_p, const float* __restrict__ beta,
                 int n_valid, int H, uint16_t* __restrict__ dH) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int k = (int)(i / H), h = (int)(i % H);
  if (k >= n_valid) return;
  const int64_t slab = (int64_t)rows_p * cols_p;
  float s = 0.f;
  for (int sp = 0; sp < k_splits; ++sp) s += partial[sp * slab + (int64_t)k * cols_p + h];
  dH[(int64_t)k * H + h] = f32_to_bf16_bits(beta[k] * s);
}

// dW tiles of a launch whose last tail_tiles tiles (in launch order) were cut into k_splits ranges of tokens:
// dW[v][h] (+)= slab 0 + slab 1 + ... of the tile, in range order.  One block per 1024 elements of a tile.
__global__ void __launch_bounds__(256)
dw_tail_reduce_kernel(const float* __restrict__ partial, GemmArgs g, int V, int H, int accumulate, float* __restrict__ dW) {
  const int pos = blockIdx.y;
  int tm, tn;
  tile_of_block(g, g.tiles_m * g.tiles_n - g.tail_tiles + pos, tm, tn);
  const float* slab = partial + (int64_t)pos * g.k_splits * (kBM * kBN);
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int e = (blockIdx.x * 4 + q) * 256 + threadIdx.x;
    const int v = tm * kBM + e / kBN, h = tn * kBN + e % kBN;
    if (v >= V || h >= H) continue;
    float sum = 0.f;
    for (int r = 0; r < g.k_splits; ++r) sum += slab[(int64_t)r * (kBM * kBN) + e];
    float* p = dW + (int64_t)v * H + h;
    *p = accumulate ? *p + sum : sum;
  }
}

// ----------------------------------------------------- reference logit ----
// ref[kk] = h_k . W[ids_k] in fp32, one wavefront per token (row-major caller arrays).
// An id outside [0, V) reads no row of W and gets the shift 0.
__global__ void __launch_bounds__(256)
target_logit_kernel(const uint16_t* __restrict__ hidden, const uint16_t* __restrict__ W, const int32_t* __restrict__ ids,
                    int n_valid, int H, int V, float* __restrict__ ref) {
  const int kk = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (kk >= n_valid) return;
  const int y = ids[kk];
  if (y < 0 || y >= V) {
    if (lane == 0) ref[kk] = 0.f;
    return;
  }
  const uint4* hp = (const uint4*)(hidden + (int64_t)kk * H);
  const uint4* wp = (const uint4*)(W + (int64_t)y * H);
  float s = 0.f;
  for (int j = lane; j < H / 8; j += 64) {
    const uint4 a = hp[j], b = wp[j];
    const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      s = fmaf(__builtin_bit_cast(float, aw[q] << 16), __builtin_bit_cast(float, bw[q] << 16), s);
      s = fmaf(__builtin_bit_cast(float, aw[q] & 0xffff0000u), __builtin_bit_cast(float, bw[q] & 0xffff0000u), s);
    }
  }
  for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
  if (lane == 0) ref[kk] = s;
}

// ------------------------------------------------- per-token statistics ----
// A granule's partial sum at or above e^70 means some numerator reached the range in which the
// clamp of the exponent shift acts (a clamped numerator alone makes its granule's sum that large).
constexpr float kShiftRangeLimit = 2.5154386709191669e30f;     // e^70

// Per-token sums of the per-granule partials: kStatTokens tokens per workgroup; the granules of a
// token are split over kStatParts groups of threads (granule gi goes to group gi % kStatParts), each
// of which walks its granules in order, and the groups' sums are added in a fixed tree, so the result
// does not depend on timing.  The walk is a chain of dependent loads: many short chains in flight hide
// their latency.  Returns to the first kStatTokens threads only.
constexpr int kStatTokens = 32, kStatParts = 8;
struct TokenSums { float S, TZ; bool in_shift_range; };
struct StatShared { float s[kStatParts][kStatTokens], t[kStatParts][kStatTokens], m[kStatParts][kStatTokens]; };

__device__ __forceinline__ TokenSums token_sums(const float* __restrict__ s_part, const float* __restrict__ t_part,
                                                int n_granules, int64_t ld, int kk, bool valid, StatShared& sh) {
  const int t = threadIdx.x % kStatTokens, part = threadIdx.x / kStatTokens;
  float s = 0.f, tz = 0.f, mx = 0.f;
  if (valid) {
#pragma unroll 8
    for (int gi = part; gi < n_granules; gi += kStatParts) {
      const float v = s_part[(int64_t)gi * ld + kk];
      s += v;
      mx = fmaxf(mx, v);
    }
    if (t_part) {
#pragma unroll 8
      for (int gi = part; gi < n_granules; gi += kStatParts) tz += t_part[(int64_t)gi * ld + kk];
    }
  }
  sh.s[part][t] = s;
  sh.t[part][t] = tz;
  sh.m[part][t] = mx;
  __syncthreads();
  TokenSums out;
  out.S = ((sh.s[0][t] + sh.s[1][t]) + (sh.s[2][t] + sh.s[3][t])) + ((sh.s[4][t] + sh.s[5][t]) + (sh.s[6][t] + sh.s[7][t]));
  out.TZ = ((sh.t[0][t] + sh.t[1][t]) + (sh.t[2][t] + sh.t[3][t])) + ((sh.t[4][t] + sh.t[5][t]) + (sh.t[6][t] + sh.t[7][t]));
  float m = sh.m[0][t];
  for (int q = 1; q < kStatParts; ++q) m = fmaxf(m, sh.m[q][t]);
  out.in_shift_range = m >= kShiftRangeLimit;
  return out;
}

__global__ void __launch_bounds__(256)
token_stats_kernel(const float* __restrict__ s_part, const float* __restrict__ t_part, int n_granules, int64_t ld,
                   const float* __restrict__ ref, const float* __restrict__ z_target, int n_valid, int chunk_start,
                   const int32_t* __restrict__ ids, int V,
                   const float* __restrict__ old_logp, const float* __restrict__ adv,
                   const int32_t* __restrict__ kept_seq, const float* __restrict__ kept_w,
                   float eps_lo, float eps_hi, float grad_scale, KlArgs klp,
                   float* __restrict__ beta_out, uint16_t* __restrict__ Eb, int kb_z,
                   float* __restrict__ logp_out, float* __restrict__ kl_out, float* __restrict__ entropy_out,
                   float* __restrict__ term, int32_t* __restrict__ diag) {
  __shared__ StatShared sh;
  const int kk = blockIdx.x * kStatTokens + threadIdx.x % kStatTokens;
  const bool valid = kk < n_valid;
  const TokenSums sums = token_sums(s_part, t_part, n_granules, ld, kk, valid, sh);
  if (threadIdx.x >= kStatTokens) return;                // the first threads finish the tokens
  bool bad_id = false, clipped = false, nonzero_adv = false;
  if (valid) {
    const float S = sums.S;
    const int k = chunk_start + kk;
    const int y = ids[kk];
    bad_id = y < 0 || y >= V;
    if (entropy_out) entropy_out[k] = logf(S) - sums.TZ / S;   // -sum_v p_v log p_v, p_v = E_v / S
    if (bad_id) {                                        // left out: no loss term, zero gradient
      beta_out[kk] = 0.f;
      if (logp_out) logp_out[k] = __builtin_nanf("");
      if (kl_out) kl_out[k] = __builtin_nanf("");
      term[k] = 0.f;
    } else {
      const float lse = ref[kk] + logf(S);
      const float logp = z_target[kk] - lse;
      const float w = kept_w[k];
      const float A = adv[kept_seq[k]];
      const TokenScalars ts = grpo_token_scalars(logp, old_logp[k], A, w, eps_lo, eps_hi, grad_scale,
                                                 klp.beta, klp.kind, klp.beta != 0.f ? klp.ref_logp[k] : 0.f);
      clipped = ts.clipped;
      nonzero_adv = A != 0.f;
      beta_out[kk] = -ts.c / S;                          // dz_kv = beta_k E_kv off the target
      // the target entry of E is replaced by E' with beta_k E' = c_k (1 - p_target): the two backward
      // contractions then need no separate one-hot term
      Eb[blk_off(kk, y, kb_z)] = f32_to_bf16_bits(-S * (1.f - __expf(logp)));
      if (logp_out) logp_out[k] = logp;
      if (kl_out) kl_out[k] = ts.kl;
      term[k] = w * ts.L;
    }
  }
  if (diag) {
    wave_count(bad_id, diag + NAT_DIAG_BAD_ID);
    wave_count(valid && sums.in_shift_range, diag + NAT_DIAG_SHIFT_RANGE);
    wave_count(clipped, diag + NAT_DIAG_CLIPPED);
    wave_count(nonzero_adv, diag + NAT_DIAG_NONZERO_ADV);
  }
}

// Forward pass alone: log-prob of the target (and the entropy) from the per-granule sums.
__global__ void __launch_bounds__(256)
logp_stats_kernel(const float* __restrict__ s_part, const float* __restrict__ t_part, int n_granules, int64_t ld,
                  const float* __restrict__ ref, const float* __restrict__ z_target, int n_valid, int chunk_start,
                  const int32_t* __restrict__ ids, int V,
                  float* __restrict__ logp_out, float* __restrict__ entropy_out, int32_t* __restrict__ diag) {
  __shared__ StatShared sh;
  const int kk = blockIdx.x * kStatTokens + threadIdx.x % kStatTokens;
  const bool valid = kk < n_valid;
  const TokenSums sums = token_sums(s_part, t_part, n_granules, ld, kk, valid, sh);
  if (threadIdx.x >= kStatTokens) return;
  bool bad_id = false;
  if (valid) {
    const int k = chunk_start + kk;
    const int y = ids[kk];
    bad_id = y < 0 || y >= V;
    logp_out[k] = bad_id ? __builtin_nanf("") : z_target[kk] - (ref[kk] + logf(sums.S));
    if (entropy_out) entropy_out[k] = logf(sums.S) - sums.TZ / sums.S;
  }
  if (diag) {
    wave_count(bad_id, diag + NAT_DIAG_BAD_ID);
    wave_count(valid && sums.in_shift_range, diag + NAT_DIAG_SHIFT_RANGE);
  }
}

// -------------------------------------------------------------- host side ----
static inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

struct Bf16Plan {
  int64_t Vp, Hp; int n_granules; int cap;      // padded vocabulary / hidden size, granules, chunk capacity (tokens)
  size_t off_Wb, off_Wtb, off_Hb, off_Hktb, off_Eb, off_s, off_t, off_zt, off_ref, off_beta, off_term, off_dh_part, total;
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
  p.off_Eb = take((size_t)cap * p.Vp * 2);      // E: rows = tokens, k = vocabulary (its one copy)
  p.off_s = take((size_t)p.n_granules * cap * 4);
  p.off_t = take((size_t)p.n_granules * cap * 4);
  p.off_zt = take((size_t)cap * 4);
  p.off_ref = take((size_t)cap * 4);
  p.off_beta = take((size_t)cap * 4);
  p.off_term = take((size_t)(N_k > 0 ? N_k : 1) * 4);
  p.off_dh_part = take((size_t)kNumCU * kBM * kBN * 4);   // raw fp32 tiles of a contraction cut into ranges (dH, or the last dW tiles): 64 MiB
  p.total = off;
  return p;
}

// Token rows per launch of the logits and dH contractions inside a chunk of `cap` rows: the smallest
// multiple of kSubChunk whose dH launch (rows / 256 x Hp / 256 tiles) fills whole waves of kNumCU
// workgroups to at least 97 %; the whole chunk if none does.  (Hp = 4096: 8192 rows = 512 tiles;
// Hp = 5120: 16384 rows = 1280 tiles; Hp = 3584 and 1024: the whole chunk.)
static int sub_chunk_rows(int cap, int Hp) {
  if (kSubChunk < 8192) return kSubChunk < cap ? kSubChunk : cap;   // a test build: the sub-chunk logic on small shapes
  const int n_col = Hp / kBN;
  for (int rows = kSubChunk; rows < cap; rows += kSubChunk) {
    const int tiles = rows / kBM * n_col;
    const int waves = (tiles + kNumCU - 1) / kNumCU;
    if (tiles * 100 >= waves * kNumCU * 97) return rows;
  }
  return cap;
}

// Chunk capacity of the recommended workspace.  Forward pass alone: kMaxChunk.  With the backward pass the
// chunk also sizes the stored soft-max numerators (cap x Vp x 2 bytes), and the dW contraction, whose
// contraction axis is the chunk, is within 0.2 % of its 32768-token speed at 16384 (measured): the
// smallest of 16384 / 24576 / 32768 rows whose dH launch fills whole rounds of workgroups to 97 %.
static int recommended_cap(int32_t N_k, int32_t H, bool backward) {
  const int64_t all = round_up(N_k > 0 ? N_k : 1, kBN);
  if (!backward) return (int)(all > kMaxChunk ? kMaxChunk : all);
  if (all <= kMaxChunk / 2) return (int)all;
  const int n_col = (int)(round_up(H, kBN) / kBN);
  for (int cap = kMaxChunk / 2; cap < kMaxChunk; cap += kMaxChunk / 4) {
    const int tiles = cap / kBM * n_col;
    const int waves = (tiles + kNumCU - 1) / kNumCU;
    if (tiles * 100 >= waves * kNumCU * 97) return (int)(all < cap ? all : cap);
  }
  return (int)(all > kMaxChunk ? kMaxChunk : all);
}

size_t loss_bf16_workspace_bytes(int32_t N_k, int32_t H, int32_t V, bool minimal) {
  return make_plan(N_k, H, V, minimal ? kBN : recommended_cap(N_k, H, true)).total;
}

// workspace of the forward pass alone: W and H_chunk blocked, the partial sums, two per-token vectors
struct FwdPlan { int64_t Vp; int n_granules; int cap; size_t off_Wb, off_Hb, off_s, off_t, off_zt, off_ref, total; };

static FwdPlan make_fwd_plan(int32_t H, int32_t V, int cap) {
  FwdPlan p;
  p.Vp = round_up(V, kBM);
  p.n_granules = (int)(p.Vp / kGranule);
  p.cap = cap;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += (bytes + 255) / 256 * 256; return o; };
  p.off_Wb = take((size_t)p.Vp * H * 2);
  p.off_Hb = take((size_t)cap * H * 2);
  p.off_s = take((size_t)p.n_granules * cap * 4);
  p.off_t = take((size_t)p.n_granules * cap * 4);
  p.off_zt = take((size_t)cap * 4);
  p.off_ref = take((size_t)cap * 4);
  p.total = off;
  return p;
}

size_t logp_bf16_workspace_bytes(int32_t N_k, int32_t H, int32_t V, bool minimal) {
  return make_fwd_plan(H, V, minimal ? kBN : recommended_cap(N_k, H, false)).total;
}

template <int NW, class Epi>
static nat_status launch_gemm(const GemmArgs& g, const Epi& epi, int prof_class, hipStream_t s) {
  ProfScope prof(prof_class, s);
  gemm_nt_kernel<Epi, NW, false><<<g.tiles_m * g.tiles_n, NW * 64, 0, s>>>(g, epi);
  NAT_LAUNCH_CHECK();
  return NAT_OK;
}

nat_status loss_bf16_run(const LossArgs& a) {
  // largest chunk capacity (multiple of 256 tokens) whose plan fits the workspace
  int cap = recommended_cap(a.N_k, a.H, true);
  while (cap > kBN && make_plan(a.N_k, a.H, a.V, cap).total > a.ws_bytes) cap -= kBN;
  const Bf16Plan p = make_plan(a.N_k, a.H, a.V, cap);
  if (p.total > a.ws_bytes) return NAT_WORKSPACE_TOO_SMALL;
  hipStream_t s = a.stream;
  char* ws = (char*)a.ws;
  uint16_t* Wb = (uint16_t*)(ws + p.off_Wb);
  uint16_t* Wtb = (uint16_t*)(ws + p.off_Wtb);
  uint16_t* Hb = (uint16_t*)(ws + p.off_Hb);
  uint16_t* Hktb = (uint16_t*)(ws + p.off_Hktb);
  uint16_t* Eb = (uint16_t*)(ws + p.off_Eb);
  float* s_part = (float*)(ws + p.off_s);
  float* t_part = a.entropy_out ? (float*)(ws + p.off_t) : nullptr;
  float* zt = (float*)(ws + p.off_zt);
  float* ref = (float*)(ws + p.off_ref);
  float* beta = (float*)(ws + p.off_beta);
  float* term = (float*)(ws + p.off_term);
  float* dh_part = (float*)(ws + p.off_dh_part);
  const uint16_t* W = (const uint16_t*)a.W;
  const uint16_t* hidden = (const uint16_t*)a.hidden;
  const int H = a.H, V = a.V;
  const int Vp = (int)p.Vp, Hp = (int)p.Hp;

  {  // W and W^T in the blocked layout, padding zero-filled
    ProfScope prof(PC_TRANSPOSE, s);
    pack_blocked_kernel<<<dim3(Vp / 64, Hp / 64), 256, 0, s>>>(W, H, V, H, Vp, Hp, Wb, Wtb, Vp / 32, nullptr);
    NAT_LAUNCH_CHECK();
  }
  const int sub = sub_chunk_rows(cap, Hp);
  for (int c0 = 0; c0 < a.N_k; c0 += cap) {
    const int nv = a.N_k - c0 < cap ? a.N_k - c0 : cap;
    const int np = (int)round_up(nv, kBN);
    const uint16_t* hid_c = hidden + (int64_t)c0 * H;
    {  // H_chunk in the blocked layout; exponent shift = target logit
      ProfScope prof(PC_TRANSPOSE, s);
      pack_blocked_kernel<<<dim3(np / 64, H / 64), 256, 0, s>>>(hid_c, H, nv, H, np, Hp, Hb, nullptr, 0, nullptr);
      NAT_LAUNCH_CHECK();
      target_logit_kernel<<<(nv + 3) / 4, 256, 0, s>>>(hid_c, W, a.ids + c0, nv, H, V, ref);
      NAT_LAUNCH_CHECK();
    }
    // The forward sweep and the dH contraction go over the chunk in sub-chunks: shorter launches of
    // the three contractions alternate, which this power-limited part rewards with a higher clock
    // (measured: both run faster on 8192 tokens than on 32768), while the dW contraction below keeps
    // the whole chunk as its contraction axis (it is the one that loses on short axes).
    for (int s0 = 0; s0 < nv; s0 += sub) {
      const int snv = nv - s0 < sub ? nv - s0 : sub;
      const int snp = (int)round_up(snv, kBN);
      uint16_t* Eb_s = Eb + (int64_t)(s0 / 256) * (Vp / 32) * kBlkElems;    // token tile s0 / 256
      const int32_t* ids_s = a.ids + c0 + s0;
      {  // logits: rows = vocabulary, columns = tokens, contraction over the hidden size
        GemmArgs g{Wb, Hb + (int64_t)(s0 / 256) * (H / 32) * kBlkElems, H, Vp / kBM, snp / kBN, NAT_GROUP_LOGITS};
        nat_status st;
        if (t_part) {
          LogitsEpilogue<true> e{V, snv, cap, Vp / 32, Eb_s, s_part + s0, t_part + s0, zt + s0, ids_s, ref + s0};
          st = launch_gemm<NAT_WAVES_LOGITS>(g, e, PC_LOGITS, s);
        } else {
          LogitsEpilogue<false> e{V, snv, cap, Vp / 32, Eb_s, s_part + s0, nullptr, zt + s0, ids_s, ref + s0};
          st = launch_gemm<NAT_WAVES_LOGITS>(g, e, PC_LOGITS, s);
        }
        if (st != NAT_OK) return st;
      }
      {
        ProfScope prof(PC_TOKEN_STATS, s);
        token_stats_kernel<<<(snv + kStatTokens - 1) / kStatTokens, kStatTokens * kStatParts, 0, s>>>(
            s_part + s0, t_part ? t_part + s0 : nullptr, p.n_granules, cap, ref + s0, zt + s0, snv, c0 + s0, ids_s, V,
            a.old_logp, a.adv, a.kept_seq, a.kept_w, a.eps_lo, a.eps_hi, a.grad_scale,
            KlArgs{a.ref_logp, a.beta_kl, a.kl_kind}, beta + s0, Eb_s, Vp / 32, a.logp, a.kl_out, a.entropy_out, term, a.diag);
        NAT_LAUNCH_CHECK();
      }
      {  // (diag(beta) H)^T of the sub-chunk into its k-slices of the chunk's blocked operand
        ProfScope prof(PC_TRANSPOSE, s);
        pack_blocked_kernel<<<dim3(snp / 64, Hp / 64), 256, 0, s>>>(hid_c + (int64_t)s0 * H, H, snv, H, snp, Hp, nullptr,
                                                                   Hktb + (int64_t)(s0 / 32) * kBlkElems, np / 32, beta + s0);
        NAT_LAUNCH_CHECK();
      }
      {  // dH: rows = tokens, columns = hidden units, contraction over the padded vocabulary
        // a launch with fewer tiles than compute units cuts the vocabulary into ranges (one workgroup per tile
        // and range, raw partial sums in fp32) and adds them up in range order afterwards
        const int tiles = (snp / kBM) * (Hp / kBN);
        int splits = tiles * 2 <= kNumCU ? kNumCU / tiles : 1;
        if (splits > 8) splits = 8;
        while (splits > 1 && (Vp / kBK) / splits < 64) --splits;
        const int kt_per = (Vp / kBK + splits - 1) / splits;
        uint16_t* dH_s = (uint16_t*)a.dH + (int64_t)(c0 + s0) * H;
        GemmArgs g{Eb_s, Wtb, Vp, snp / kBM, Hp / kBN, NAT_GROUP_DHIDDEN, 0, splits, kt_per};
        DHiddenEpilogue e{snv, H, dH_s, beta + s0, splits > 1 ? dh_part : nullptr, snp, Hp};
        {
          ProfScope prof(PC_DHIDDEN, s);
          gemm_nt_kernel<DHiddenEpilogue, NAT_WAVES_DHIDDEN, false><<<tiles * splits, NAT_WAVES_DHIDDEN * 64, 0, s>>>(g, e);
          NAT_LAUNCH_CHECK();
          if (splits > 1) {
            const int64_t n = (int64_t)snv * H;
            dh_reduce_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(dh_part, splits, snp, Hp, beta + s0, snv, H, dH_s);
            NAT_LAUNCH_CHECK();
          }
        }
      }
    }
    {  // dW: rows = vocabulary, columns = hidden units, contraction over the chunk's (padded) tokens
      // A = E from its one copy (rows = token), i.e. stored along this contraction's k axis
      // The tiles left over after the last full round of one tile per compute unit would occupy a fraction
      // of the chip for a whole tile time: their token axis is cut into ranges (one workgroup per tile and
      // range, raw sums to slabs) that are added into dW in range order afterwards.
      const int tiles = (Vp / kBM) * (Hp / kBN), kt_all = np / kBK;
      const int tail = tiles % kNumCU;
      int splits = (tail > 0 && tail * 2 <= kNumCU) ? kNumCU / tail : 1, kt_per = kt_all;
      if (splits > 8) splits = 8;
      while (splits > 1 && kt_all / splits < kMinSlicesPerRange) --splits;
      if (splits > 1) {
        kt_per = (int)round_up((kt_all + splits - 1) / splits, 8);
        splits = (kt_all + kt_per - 1) / kt_per;               // every range non-empty
      }
      const int accumulate = (c0 > 0 || a.accumulate_dw) ? 1 : 0;
      GemmArgs g{Eb, Hktb, np, Vp / kBM, Hp / kBN, NAT_GROUP_DWEIGHT, Vp / 32, splits, kt_per, splits > 1 ? tail : 0};
      DWeightEpilogue e{V, H, accumulate, a.dW, dh_part};
      {
        ProfScope prof(PC_DWEIGHT, s);
        const int grid = splits > 1 ? tiles - tail + tail * splits : tiles;
        gemm_nt_kernel<DWeightEpilogue, NAT_WAVES_DWEIGHT, true><<<grid, NAT_WAVES_DWEIGHT * 64, 0, s>>>(g, e);
        NAT_LAUNCH_CHECK();
        if (splits > 1) {
          dw_tail_reduce_kernel<<<dim3(kBM * kBN / 1024, tail), 256, 0, s>>>(dh_part, g, V, H, accumulate, a.dW);
          NAT_LAUNCH_CHECK();
        }
      }
    }
  }
  ProfScope prof(PC_LOSS_REDUCE, s);
  loss_reduce_kernel<<<1, 1024, 0, s>>>(term, a.N_k, a.loss);
  NAT_LAUNCH_CHECK();
  return NAT_OK;
}

nat_status logp_bf16_run(const LogpArgs& a) {
  int cap = recommended_cap(a.N_k, a.H, false);
  while (cap > kBN && make_fwd_plan(a.H, a.V, cap).total > a.ws_bytes) cap -= kBN;
  const FwdPlan p = make_fwd_plan(a.H, a.V, cap);
  if (p.total > a.ws_bytes) return NAT_WORKSPACE_TOO_SMALL;
  hipStream_t s = a.stream;
  char* ws = (char*)a.ws;
  uint16_t* Wb = (uint16_t*)(ws + p.off_Wb);
  uint16_t* Hb = (uint16_t*)(ws + p.off_Hb);
  float* s_part = (float*)(ws + p.off_s);
  float* t_part = a.entropy ? (float*)(ws + p.off_t) : nullptr;
  float* zt = (float*)(ws + p.off_zt);
  float* ref = (float*)(ws + p.off_ref);
  const uint16_t* W = (const uint16_t*)a.W;
  const uint16_t* hidden = (const uint16_t*)a.hidden;
  const int H = a.H, V = a.V, Vp = (int)p.Vp;
  {
    ProfScope prof(PC_TRANSPOSE, s);
    pack_blocked_kernel<<<dim3(Vp / 64, H / 64), 256, 0, s>>>(W, H, V, H, Vp, H, Wb, nullptr, 0, nullptr);
    NAT_LAUNCH_CHECK();
  }
  for (int c0 = 0; c0 < a.N_k; c0 += cap) {
    const int nv = a.N_k - c0 < cap ? a.N_k - c0 : cap;
    const int np = (int)round_up(nv, kBN);
    const uint16_t* hid_c = hidden + (int64_t)c0 * H;
    {
      ProfScope prof(PC_TRANSPOSE, s);
      pack_blocked_kernel<<<dim3(np / 64, H / 64), 256, 0, s>>>(hid_c, H, nv, H, np, H, Hb, nullptr, 0, nullptr);
      NAT_LAUNCH_CHECK();
      target_logit_kernel<<<(nv + 3) / 4, 256, 0, s>>>(hid_c, W, a.ids + c0, nv, H, V, ref);
      NAT_LAUNCH_CHECK();
    }
    {
      GemmArgs g{Wb, Hb, H, Vp / kBM, np / kBN, NAT_GROUP_LOGITS};
      nat_status st;
      if (t_part) {
        LogitsEpilogue<true, false> e{V, nv, cap, 0, nullptr, s_part, t_part, zt, a.ids + c0, ref};
        st = launch_gemm<NAT_WAVES_LOGITS>(g, e, PC_LOGITS, s);
      } else {
        LogitsEpilogue<false, false> e{V, nv, cap, 0, nullptr, s_part, nullptr, zt, a.ids + c0, ref};
        st = launch_gemm<NAT_WAVES_LOGITS>(g, e, PC_LOGITS, s);
      }
      if (st != NAT_OK) return st;
    }
    {
      ProfScope prof(PC_TOKEN_STATS, s);
      logp_stats_kernel<<<(nv + kStatTokens - 1) / kStatTokens, kStatTokens * kStatParts, 0, s>>>(s_part, t_part, p.n_granules, cap, ref, zt, nv, c0, a.ids + c0, V,
                                                      a.logp, a.entropy, a.diag);
      NAT_LAUNCH_CHECK();
    }
  }
  return NAT_OK;
}

}  // namespace nat
