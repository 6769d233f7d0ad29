/*
 * nat.h -- C ABI of the partial-token GRPO loss stage of NAT ("Not All Tokens
 * are Needed") for AMD MI355X (gfx950).
 *
 * Path:  rewards -> nat_advantage -> nat_select -> nat_compact -> nat_loss_fwd_bwd
 * Around it: nat_select_schedule / nat_select_poisson + nat_compact_pi (other selection
 * laws inside the same estimator), nat_prefix_pack (the truncated batch for the model
 * body), nat_loss_fwd_bwd_kl (token loss with the KL term, entropy), nat_logp_fwd (the
 * forward pass alone).
 *
 * Notation follows the paper: P prompts, G rollouts per prompt, B = P*G
 * rollouts, T_i response length of rollout i, t = 1..T_i token position,
 * m_{i,t} selection mask, p_{i,t} inclusion probability, L_i RPC cut point,
 * C minimum retained prefix, A_i group-relative advantage, r_{i,t} importance
 * ratio, S_{i,t} clipped surrogate.  Response tokens of all rollouts are
 * packed back to back: token (i, t) sits at packed position
 * cu_seqlens[i] + (t - 1); N = cu_seqlens[B] tokens in total, N_k kept.
 *
 * Conventions
 *   - every pointer named d_* is DEVICE memory, h_* is HOST memory;
 *   - the library never allocates or frees device memory: all buffers,
 *     including workspaces, belong to the caller (query the *_workspace_bytes
 *     functions);
 *   - all work is enqueued on the caller's stream (`stream` is a hipStream_t
 *     passed as void*; NULL = the default stream); no call synchronises with
 *     the host;
 *   - outputs are fully overwritten unless stated otherwise;
 *   - every function returns a nat_status and never throws; argument errors
 *     are detected on the host before anything is launched;
 *   - values that live in device memory cannot be checked by the host.  The
 *     kernels bound every access they derive from them: packed positions at or
 *     beyond cu_seqlens[B] (when the host-passed N is larger) are never kept,
 *     offsets beyond N are clamped to N, the kept-token outputs are written only
 *     below their stated capacity, and token ids outside [0, V) are skipped and
 *     counted (see nat_loss_fwd_bwd_kl).
 */
#ifndef NAT_H_
#define NAT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t nat_status;
enum {
  NAT_OK = 0,
  NAT_INVALID_ARG = 1,          /* NULL required pointer, parameter out of range      */
  NAT_BAD_SHAPE = 2,            /* size not supported by the kernels                   */
  NAT_WORKSPACE_TOO_SMALL = 3,
  NAT_UNSUPPORTED_DTYPE = 4,
  NAT_HIP_ERROR = 5             /* a HIP runtime call failed (launch, copy, event)     */
};

enum { NAT_SCHEME_FULL = 0, NAT_SCHEME_URS = 1, NAT_SCHEME_RPC = 2, NAT_SCHEME_DET = 3 };
enum { NAT_DTYPE_F32 = 0, NAT_DTYPE_BF16 = 1 };
/* sampled-token forms of the KL term of Eq. 4, with d = ref_logp - logp:
 * LOG_RATIO: -d (the form named in the footnote to Eq. 4);  NONNEG: exp(d) - d - 1. */
enum { NAT_KL_LOG_RATIO = 0, NAT_KL_NONNEG = 1 };
/* words of the optional diagnostic array of nat_loss_fwd_bwd_kl / nat_logp_fwd */
enum { NAT_DIAG_BAD_ID = 0, NAT_DIAG_SHIFT_RANGE = 1, NAT_DIAG_CLIPPED = 2, NAT_DIAG_NONZERO_ADV = 3,
       NAT_DIAG_WORDS = 4 };

/* Human-readable name of a status code (static string, never NULL). */
const char* nat_status_string(nat_status s);

/*
 * Selection parameters (Sec. 3.1 and Sec. 4 of the paper).
 *   scheme      FULL: every token, p_{i,t} = 1 (full-token GRPO, Eq. 5).
 *               URS:  m_{i,t} ~ Bernoulli(p) i.i.d., p_{i,t} = p (Sec. 3.1).
 *               RPC:  L_i ~ Uniform{C_i..T_i}, C_i = min(max(C,1),T_i),
 *                     m_{i,t} = 1{t <= L_i} (Eq. 7), p_{i,t} = 1 for t <= C_i and
 *                     (T_i-t+1)/(T_i-C_i+1) after (Eq. 8; Sec. 4 "Minimum-cutoff RPC").
 *               DET:  keep the first K_i = floor(trunc_frac*T_i) tokens, weight as if
 *                     p = 1 (the biased control of Sec. 4).
 *   Random bits: Philox4x32-10, key = (seed low, seed high), counter =
 *   (t0 >> 2, rollout_id_base + i, stream, step) with t0 = t - 1; stream 0 = URS
 *   token draws (word t0 & 3 of the block; keep iff word < floor(p * 2^32)),
 *   stream 1 = RPC cut (word 0; L_i = C_i + ((word * n) >> 32), n = T_i-C_i+1).
 *   A draw depends only on (seed, step, global rollout id, t), so it does not
 *   change with batching or sharding.
 *   d_scheme_per_rollout: optional DEVICE array [B] overriding `scheme` per
 *   rollout (mixed batches); NULL = uniform scheme.
 *   d_drop_zero_adv: see the field; honoured by nat_select, nat_select_schedule and
 *   nat_select_poisson (inclusion probabilities and weights of the other rollouts do not change).
 */
typedef struct nat_select_params {
  int32_t scheme;
  int32_t min_cut;           /* C >= 1 (RPC)                       */
  double p;                  /* URS keep probability, in (0, 1]    */
  double trunc_frac;         /* DET fraction beta, in (0, 1]       */
  uint64_t seed;
  uint32_t step;
  int32_t rollout_id_base;   /* global id of rollout 0 of this batch */
  const int32_t* d_scheme_per_rollout;
  const float* d_drop_zero_adv;   /* optional DEVICE array [B] of advantages (Eq. 2): rollouts whose advantage
                                     is exactly 0 keep nothing (cut_len 0).  With A = 0, Eq. 3 gives S = 0 and a
                                     zero gradient at every token, so the estimate is unchanged as long as the
                                     token loss has no KL term; NULL = keep the paper's behaviour */
} nat_select_params;

/*
 * Group-relative advantage, Eq. 2:  A = (R - mean) / (std + eps_adv) with the
 * population standard deviation over the G rollouts of each prompt.
 *   d_rewards [P*G] float32 (prompt-major), d_adv [P*G] float32 out.
 * Errors: NULL pointer, P <= 0, G <= 0, eps_adv < 0 -> NAT_INVALID_ARG.
 */
nat_status nat_advantage(const float* d_rewards, int32_t P, int32_t G, float eps_adv,
                         float* d_adv, void* stream);

/* Number of uint32 words of the packed mask of N tokens: 2 * ceil(N / 64). */
int64_t nat_mask_words(int64_t N);

/*
 * Draw the selection mask (Sec. 3.1 "Random masking", Eq. 7).
 *   d_cu_seqlens [B+1] int64, non-decreasing, cu_seqlens[0] = 0, cu_seqlens[B] = N
 *                (the host passes N so that no read-back is needed);
 *   d_cut_len    [B] int32 out: L_i (RPC), K_i (DET), T_i (FULL, URS);
 *   d_mask_bits  [nat_mask_words(N)] uint32 out: bit (n & 31) of word n >> 5 is the
 *                mask of packed position n; bits at positions >= N are zero.
 * Errors: NULL pointer, B <= 0, N < 0 or N >= 2^31, unknown scheme, p outside (0,1],
 * min_cut < 1, trunc_frac outside (0,1] -> NAT_INVALID_ARG.  N = 0 is valid.
 */
nat_status nat_select(const nat_select_params* params, const int64_t* d_cu_seqlens, int32_t B,
                      int64_t N, int32_t* d_cut_len, uint32_t* d_mask_bits, void* stream);

/* Bytes of device workspace nat_compact needs for N tokens. */
size_t nat_compact_workspace_bytes(int64_t N);

/*
 * Stable mask -> index compaction with the Horvitz-Thompson weight of every
 * kept token (Eq. 6 / Eq. 9 folded with the 1/G * 1/|o_i| averaging of Eq. 5):
 *     kept_w = 1 / (n_rollouts_global * T_i * p_{i,t})   (one fp64 division, rounded to fp32)
 * with p_{i,t} recomputed from (scheme, p, C, T_i, t) of `params`.
 *   kept_cap   capacity, in kept tokens, of every per-kept-token output below (N always
 *              suffices; a caller that knows a tighter bound may pass less).  Entries at
 *              index >= kept_cap are not written; d_n_kept still reports the true count,
 *              so n_kept > kept_cap tells the caller that the outputs are truncated;
 *   d_kept_idx [kept_cap] int32 out: packed positions of kept tokens, ascending;
 *   d_kept_seq [kept_cap] int32 out: rollout index i of each kept token;
 *   d_kept_w   [kept_cap] float out;
 *   d_cu_kept  [B+1] int32 out: kept-token offsets per rollout;
 *   d_n_kept   [1] int32 out;  h_n_kept: optional PINNED host int32 that receives the
 *              same value by an asynchronous copy on `stream` (NULL = skip);
 *   optional gather (any of the three pairs may be NULL):
 *     d_hidden [N, H] -> d_hidden_k [kept_cap, H] rows of kept tokens, dtype NAT_DTYPE_*,
 *     d_ids [N] -> d_ids_k [kept_cap],  d_old_logp [N] -> d_old_logp_k [kept_cap];
 *   d_ws / ws_bytes: workspace of at least nat_compact_workspace_bytes(N).
 * Errors: as nat_select, plus n_rollouts_global <= 0, kept_cap < 0 -> NAT_INVALID_ARG; H <= 0
 * or a row size that is not a multiple of 16 bytes when gathering -> NAT_BAD_SHAPE, d_hidden /
 * d_hidden_k not 16-byte aligned -> NAT_INVALID_ARG, workspace too small.
 */
nat_status nat_compact(const nat_select_params* params, int32_t n_rollouts_global,
                       const uint32_t* d_mask_bits, const int64_t* d_cu_seqlens, int32_t B, int64_t N,
                       int64_t kept_cap, int32_t* d_kept_idx, int32_t* d_kept_seq, float* d_kept_w, int32_t* d_cu_kept,
                       int32_t* d_n_kept, int32_t* h_n_kept,
                       const void* d_hidden, void* d_hidden_k, int32_t H, int32_t dtype,
                       const int32_t* d_ids, int32_t* d_ids_k,
                       const float* d_old_logp, float* d_old_logp_k,
                       void* d_ws, size_t ws_bytes, void* stream);

/*
 * nat_compact for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same
 * arguments (minus the workspace), same kernels and bit-identical outputs; the tile counts and
 * offsets live in a scratch array that is part of the library's device image (about 513 KiB,
 * resident on each GPU the library is used on until the process ends).  The call itself
 * allocates and frees nothing, on the device or through any runtime routine, and never creates
 * timing events (nat_profile_enable does not see it).
 *   N may not exceed NAT_COMPACT_STATIC_MAX_TOKENS -> NAT_BAD_SHAPE.
 *   The device is the one current on the calling thread; `stream` must belong to it.
 *   All calls on one GPU share that GPU's scratch: calls that overlap in time on one GPU
 *   (different streams, different threads) race and give undefined results; calls ordered by
 *   a stream or by events are fine, and nothing needs clearing in between.
 * Other errors: as nat_compact; a failing symbol lookup -> NAT_HIP_ERROR.
 */
#define NAT_COMPACT_STATIC_MAX_TOKENS 268435456   /* 2^28 */
nat_status nat_compact_static(const nat_select_params* params, int32_t n_rollouts_global,
                              const uint32_t* d_mask_bits, const int64_t* d_cu_seqlens, int32_t B, int64_t N,
                              int64_t kept_cap, int32_t* d_kept_idx, int32_t* d_kept_seq, float* d_kept_w,
                              int32_t* d_cu_kept, int32_t* d_n_kept, int32_t* h_n_kept,
                              const void* d_hidden, void* d_hidden_k, int32_t H, int32_t dtype,
                              const int32_t* d_ids, int32_t* d_ids_k,
                              const float* d_old_logp, float* d_old_logp_k, void* stream);

/*
 * Cut every rollout by its own cut-length distribution (Sec. 4, Eq. 7-8: L_i ~ q_i,
 * mask 1{t <= L_i}, survival p_{i,t} = sum_{l >= t} q_i(l)).
 *   d_weights [N] uint32: non-negative integer weights a_{i,l}, one per response
 *             position, packed like the tokens; q_i(l) = a_{i,l} / A_i, A_i = sum_l a_{i,l}.
 *             The last weight of a rollout should be positive so that p_{i,T_i} > 0.
 *             A rollout whose weights are all zero is kept whole with p = 1.
 *   The cut is the first l whose running sum exceeds r = (u64 * A_i) >> 64, u64 built
 *   from two words of one Philox block (stream 2) keyed by (seed, step, global rollout
 *   id); only seed, step and rollout_id_base of `params` are read.
 *   d_cut_len [B] int32 out: L_i;  d_mask_bits as in nat_select;
 *   d_pi      [N] double out: p_{i,t} = (sum_{l >= t} a_{i,l}) / A_i for EVERY position, kept
 *             or not: one fp64 division of the two integers, each converted to fp64 with
 *             round-to-nearest-even.  Both are exact while A_i < 2^53 (any rollout shorter
 *             than 2^21 tokens); beyond that (A_i can reach 2^63) each carries a relative
 *             rounding error of at most 2^-53 before the division.  The cut itself is
 *             always drawn in exact 64-bit integer arithmetic.
 * Errors: NULL pointer, B <= 0, N < 0 or N >= 2^31 -> NAT_INVALID_ARG.
 */
nat_status nat_select_schedule(const nat_select_params* params, const uint32_t* d_weights,
                               const int64_t* d_cu_seqlens, int32_t B, int64_t N,
                               int32_t* d_cut_len, uint32_t* d_mask_bits, double* d_pi, void* stream);

/*
 * Independent masks m_{i,t} ~ Bernoulli(p_{i,t}) with caller-supplied, token-dependent
 * inclusion probabilities (Sec. 3.1 "Random masking"; the information-aware extension
 * named in the discussion section).
 *   d_pi [N] double in [0,1]: keep iff u32 < floor(p * 2^32), with the same random words
 *        as NAT_SCHEME_URS (a constant p reproduces URS exactly).  Values <= 0 (or NaN)
 *        never keep, values >= 1 always keep.  Tokens with p = 0 make the estimator
 *        biased (Prop. 1 needs p > 0): that is the caller's choice.
 * Only seed, step and rollout_id_base of `params` are read.  Errors as nat_select_schedule.
 */
nat_status nat_select_poisson(const nat_select_params* params, const double* d_pi,
                              const int64_t* d_cu_seqlens, int32_t B, int64_t N,
                              uint32_t* d_mask_bits, void* stream);

/*
 * nat_compact for masks drawn with explicit inclusion probabilities (nat_select_schedule,
 * nat_select_poisson): identical outputs, but the weight of Eq. 6 / Eq. 9 is
 *     kept_w = 1 / ((n_rollouts_global * T_i) * d_pi[n])
 * (integer product, one fp64 multiplication, one fp64 division, rounded to fp32).
 * Workspace: nat_compact_workspace_bytes(N).  Errors as nat_compact.
 */
nat_status nat_compact_pi(int32_t n_rollouts_global, const uint32_t* d_mask_bits, const double* d_pi,
                          const int64_t* d_cu_seqlens, int32_t B, int64_t N,
                          int64_t kept_cap, int32_t* d_kept_idx, int32_t* d_kept_seq, float* d_kept_w, int32_t* d_cu_kept,
                          int32_t* d_n_kept, int32_t* h_n_kept,
                          const void* d_hidden, void* d_hidden_k, int32_t H, int32_t dtype,
                          const int32_t* d_ids, int32_t* d_ids_k,
                          const float* d_old_logp, float* d_old_logp_k,
                          void* d_ws, size_t ws_bytes, void* stream);

/*
 * Truncated batch for a model body that runs only over the kept prefixes (Sec. 4, the
 * paragraph on compute savings): rollout i becomes its P_i prompt tokens followed by its
 * first L_i response tokens.
 *   d_prompt_len [B] int32 or NULL (no prompts: P_i = 0);
 *   d_cu_seqlens [B+1] int64 response-token offsets as in nat_select;
 *   d_cut_len    [B] int32 from nat_select / nat_select_schedule (values outside [0, T_i]
 *                are clamped);
 *   next_token_shift: 1 = the row that scores response token t is the row before it
 *                (next-token prediction; every P_i must be >= 1), 0 = its own row;
 *   rows_cap:    capacity of the per-row outputs; sum_i (P_i + T_i) always suffices;
 *   d_cu_packed  [B+1] int32 out: row offsets of the truncated sequences;
 *   d_cu_loss    [B+1] int32 out: offsets of the kept response tokens (= sum of L_j);
 *   d_src_idx    [rows_cap] int32 out: for each truncated row, its row in the full packed
 *                input (prompt and response of rollout 0, then of rollout 1, ...);
 *   d_position_ids [rows_cap] int32 out: 0 .. P_i + L_i - 1 within each sequence;
 *   d_loss_row   [kept_cap] int32 out: truncated row whose output scores kept response
 *                token k (ascending (i, t), the order of nat_compact); kept_cap >= sum L_i
 *                (N always suffices);
 *   d_totals     [2] int32 out: number of truncated rows, longest truncated sequence;
 *   h_totals     optional PINNED host int32[2] receiving the same by an asynchronous copy;
 *   d_input_ids -> d_input_ids_packed: optional gather of the full input's token ids
 *                ([sum_i (P_i + T_i)] -> [rows_cap]); both NULL to skip.
 * Rows beyond rows_cap / kept_cap are not written.
 * Errors: NULL required pointer, B <= 0, rows_cap < 0, kept_cap < 0, shift not 0/1,
 * shift = 1 without prompt lengths -> NAT_INVALID_ARG.
 */
nat_status nat_prefix_pack(const int32_t* d_prompt_len, const int64_t* d_cu_seqlens,
                           const int32_t* d_cut_len, int32_t B, int32_t next_token_shift,
                           int64_t rows_cap, int64_t kept_cap,
                           int32_t* d_cu_packed, int32_t* d_cu_loss, int32_t* d_src_idx,
                           int32_t* d_position_ids, int32_t* d_loss_row, int32_t* d_totals,
                           int32_t* h_totals, const int32_t* d_input_ids, int32_t* d_input_ids_packed,
                           void* stream);

/*
 * Forward pass alone: log-probability of given tokens under the head (the evaluation that
 * produces behaviour and reference log-probs; Sec. 2, cost structure of a GRPO step, stage 2),
 * and optionally the entropy of each row:
 *     z_k = W h_k,  logp_k = z_k[ids_k] - logsumexp(z_k),  entropy_k = -sum_v p_v log p_v.
 * Same projection kernel and the same arithmetic as nat_loss_fwd_bwd (identical log-probs for
 * identical chunking), but no soft-max numerators are written: 2 V H flops per token.
 *   d_hidden_k [N_k, H], d_W [V, H] row-major (bf16 or f32), d_ids_k [N_k] int32 in [0, V);
 *   d_logp_k [N_k] float out;  d_entropy_k [N_k] float out or NULL;
 *   d_diag   [NAT_DIAG_WORDS] int32 out or NULL: NAT_DIAG_BAD_ID and NAT_DIAG_SHIFT_RANGE as
 *            described at nat_loss_fwd_bwd_kl (the other words are set to 0); a token whose id
 *            lies outside [0, V) gets log-prob NaN;
 *   d_ws / ws_bytes: at least nat_logp_workspace_min_bytes (nat_logp_workspace_bytes recommended).
 * The bf16 path shifts exponents by the target logit: as for nat_loss_fwd_bwd, log(p_max/p_target)
 * must stay below 70 (tokens beyond it are counted in d_diag).  N_k = 0 is valid and does nothing
 * but clear d_diag.
 * Errors and alignment: as nat_loss_fwd_bwd.
 */
size_t nat_logp_workspace_bytes(int32_t N_k, int32_t H, int32_t V, int32_t dtype);
size_t nat_logp_workspace_min_bytes(int32_t N_k, int32_t H, int32_t V, int32_t dtype);
nat_status nat_logp_fwd(const void* d_hidden_k, const void* d_W, const int32_t* d_ids_k,
                        int32_t N_k, int32_t H, int32_t V, int32_t dtype,
                        float* d_logp_k, float* d_entropy_k, int32_t* d_diag,
                        void* d_ws, size_t ws_bytes, void* stream);

/*
 * Workspace for nat_loss_fwd_bwd.  *_bytes is the recommended size (largest
 * token chunk the kernels use); *_min_bytes the smallest size accepted (one
 * token tile per chunk).  Both return 0 for unsupported arguments.
 */
size_t nat_loss_workspace_bytes(int32_t N_k, int32_t H, int32_t V, int32_t dtype);
size_t nat_loss_workspace_min_bytes(int32_t N_k, int32_t H, int32_t V, int32_t dtype);

/*
 * LM-head projection, full-vocabulary log-softmax, clipped-ratio GRPO surrogate
 * and its gradients on the kept tokens (Eq. 1, Eq. 3, Eq. 5, Eq. 6/9; App. A):
 *     z_k = W h_k,  logp_k = z_k[ids_k] - logsumexp(z_k),
 *     r_k = exp(logp_k - old_logp_k),  A = adv[kept_seq[k]],
 *     S_k = min(r_k A, clip(r_k, 1-eps_lo, 1+eps_hi) A),
 *     loss = - sum_k kept_w[k] S_k                     (the paper maximises J; loss = -J_hat)
 *     c_k = -grad_scale * kept_w[k] * dS_k/dlogp_k,  dS/dlogp = r A if (A>0 and r<=1+eps_hi)
 *                                                     or (A<0 and r>=1-eps_lo), else 0,
 *     dz_k = c_k (onehot(ids_k) - softmax(z_k)),  dH_k = W^T dz_k,  dW = sum_k dz_k h_k^T.
 * The KL term of Eq. 4 is not included (beta = 0 as in Sec. 5.1); see nat_loss_fwd_bwd_kl.
 *   d_hidden_k [N_k, H] row-major, dtype bf16 or f32;  d_W [V, H] row-major, same dtype;
 *   d_ids_k [N_k] int32 in [0, V);  d_old_logp_k [N_k] float;  d_adv [>= max(kept_seq)+1] float;
 *   d_loss [1] float out;  d_logp_k [N_k] float out or NULL;
 *   d_dH_k [N_k, H] out, same dtype as the inputs;
 *   d_dW [V, H] float32 out: overwritten, or added to when accumulate_dw != 0.  Ordinary device memory
 *     (hipMalloc or a sub-range of it), not host-coherent / fine-grained memory: chunks after the first are
 *     added with the GPU's fp32 memory atomics (one addition per element and chunk, chunks in stream order).
 *   The reduction order of d_dW and d_loss is fixed: results are bit-identical from run to run.
 *   The [N_k, V] logits are never written to memory as a whole; the bf16 path keeps the bf16
 *   soft-max numerators exp(z - z_target) of one token chunk (16384 tokens with the recommended
 *   workspace, 32768 for hidden sizes whose dH launch would not fill whole rounds of workgroups at
 *   16384; fewer with a smaller workspace) in the workspace.  That shift requires log(p_max / p_target) < 70 for every kept token (larger
 *   numerators are clamped; nat_loss_fwd_bwd_kl counts the tokens this may have touched); the
 *   fp32 path has no such bound.  A token whose id lies outside [0, V) is left out of loss, dH
 *   and dW (nat_loss_fwd_bwd_kl counts those too).
 * N_k = 0 is valid: loss = 0, d_dW zeroed unless accumulating, d_dH_k untouched.
 *   Alignment: d_hidden_k, d_W, d_dH_k, d_dW 16 bytes; d_ws 256 bytes (else NAT_INVALID_ARG).
 * Errors: NULL pointer, N_k < 0, eps < 0 -> NAT_INVALID_ARG; H <= 0, V <= 0, or (bf16) H not
 * a multiple of 64 -> NAT_BAD_SHAPE; dtype unknown -> NAT_UNSUPPORTED_DTYPE; ws_bytes below
 * nat_loss_workspace_min_bytes -> NAT_WORKSPACE_TOO_SMALL.
 */
nat_status nat_loss_fwd_bwd(const void* d_hidden_k, const void* d_W, const int32_t* d_ids_k,
                            const float* d_old_logp_k, const float* d_adv, const int32_t* d_kept_seq,
                            const float* d_kept_w, int32_t N_k, int32_t H, int32_t V, int32_t dtype,
                            float eps_lo, float eps_hi, float grad_scale,
                            float* d_loss, float* d_logp_k, void* d_dH_k, float* d_dW,
                            int32_t accumulate_dw, void* d_ws, size_t ws_bytes, void* stream);

/*
 * nat_loss_fwd_bwd with the token loss of Eq. 4, L_k = S_k - beta_kl * KL_k, and two
 * per-token diagnostics.  KL_k is a sampled-token estimate of D_KL(pi_theta || pi_ref)
 * computed from d_k = d_ref_logp_k[k] - logp_k in the form `kl_kind` (NAT_KL_*):
 *     loss = - sum_k kept_w[k] (S_k - beta_kl KL_k),
 *     c_k  = -grad_scale * kept_w[k] * (dS_k/dlogp_k - beta_kl dKL_k/dlogp_k),
 * everything else as nat_loss_fwd_bwd (same kernels; beta_kl = 0 gives the same bits).
 *   d_ref_logp_k [N_k] float: log-probability of the sampled token under the reference
 *                policy; may be NULL when beta_kl = 0;
 *   d_kl_k       [N_k] float out or NULL: KL_k (0 when beta_kl = 0);
 *   d_entropy_k  [N_k] float out or NULL: -sum_v p_v log p_v of the current policy at each
 *                kept token (the quantity of the paper's entropy curves), accumulated in the
 *                same sweep over the vocabulary; it has no gradient.
 *   d_diag       [NAT_DIAG_WORDS] int32 out or NULL: counters over the kept tokens of this call
 *                (cleared first, exact, independent of scheduling):
 *                  NAT_DIAG_BAD_ID       tokens whose id lies outside [0, V).  Such a token is
 *                                        left out: no contribution to loss, dH (its row is 0) or
 *                                        dW; its log-prob and KL are reported as NaN;
 *                  NAT_DIAG_SHIFT_RANGE  (bf16 path) tokens for which some 128-row block of the
 *                                        vocabulary has numerators summing to e^70 or more, i.e.
 *                                        log(p_max / p_target) reached the range where the clamp
 *                                        of the exponent shift may have acted: their log-probs
 *                                        and gradients are not reliable.  Always 0 on the fp32
 *                                        path, which shifts by the row maximum;
 *                  NAT_DIAG_CLIPPED      tokens with A != 0 whose surrogate gradient is zero
 *                                        because the ratio left [1 - eps_lo, 1 + eps_hi] on the
 *                                        side that Eq. 3 clips (the clipping frequency of the
 *                                        paper's App. C figure is CLIPPED / NONZERO_ADV);
 *                  NAT_DIAG_NONZERO_ADV  tokens with A != 0.
 * Errors: as nat_loss_fwd_bwd, plus beta_kl < 0, unknown kl_kind, or beta_kl > 0 with
 * d_ref_logp_k NULL -> NAT_INVALID_ARG.
 */
nat_status nat_loss_fwd_bwd_kl(const void* d_hidden_k, const void* d_W, const int32_t* d_ids_k,
                               const float* d_old_logp_k, const float* d_adv, const int32_t* d_kept_seq,
                               const float* d_kept_w, int32_t N_k, int32_t H, int32_t V, int32_t dtype,
                               float eps_lo, float eps_hi, float grad_scale,
                               const float* d_ref_logp_k, float beta_kl, int32_t kl_kind,
                               float* d_loss, float* d_logp_k, float* d_kl_k, float* d_entropy_k,
                               int32_t* d_diag, void* d_dH_k, float* d_dW, int32_t accumulate_dw,
                               void* d_ws, size_t ws_bytes, void* stream);

/*
 * Per-kernel timing (measurement aid, off by default).  When enabled, every
 * kernel launch of the library is bracketed by a pair of HIP events on the
 * caller's stream.  nat_profile_collect waits for those events, adds the elapsed
 * milliseconds and launch counts per kernel class into the caller's HOST arrays
 * (length n_classes = nat_profile_num_classes()) and clears the record.
 */
int32_t nat_profile_num_classes(void);
const char* nat_profile_class_name(int32_t cls);
nat_status nat_profile_enable(int32_t on);
nat_status nat_profile_collect(double* h_ms, int64_t* h_launches, int32_t n_classes);

/*
 * Practical ceilings of the machine (measurement aids, not on the path).  The caller times them
 * with events on `stream`.
 *   nat_probe_mfma_bf16: 2048 workgroups of 4 wavefronts, each issuing `iters` x 16 independent
 *     32x32x16 bf16 matrix products on operands held in registers (random_operands = 0: constant
 *     operands; 1: pseudo-random sign and mantissa bits, which is what the power limit sees on
 *     real data).  d_scratch: nat_probe_mfma_scratch_bytes() of device memory (written, contents
 *     meaningless); *h_flops (HOST, may be NULL) receives the flops of the launch.
 *   nat_probe_copy: copies `bytes` (a multiple of 16; both pointers 16-byte aligned) with 16-byte
 *     loads and stores: 2 * bytes of HBM traffic of known size.
 * Errors: NULL pointer, iters <= 0, misaligned or odd-sized copy -> NAT_INVALID_ARG.
 */
size_t nat_probe_mfma_scratch_bytes(void);
nat_status nat_probe_mfma_bf16(int32_t random_operands, int32_t iters, float* d_scratch,
                               double* h_flops, void* stream);
nat_status nat_probe_copy(void* d_dst, const void* d_src, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* NAT_H_ */
