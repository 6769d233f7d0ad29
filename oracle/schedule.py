"""General cut-length schedules, Poisson sampling with given inclusion
probabilities, and prefix packing.

Follows Sec. 4: a cut L_i in {1..T_i} drawn from any distribution q_i(l), the
mask 1{t <= L_i}, the survival function p_{i,t} = sum_{l >= t} q_i(l) (Eq. 7-8)
and the estimator of Eq. 9; Sec. 3.1: independent m_{i,t} ~ Bernoulli(p_{i,t})
with arbitrary p_{i,t} > 0 and the estimator of Eq. 6 (the discussion section
names token-dependent probabilities inside the same Horvitz-Thompson form as
the extension); and the compute-savings paragraph of Sec. 4: the model body
only has to run over the first L_i response tokens of each rollout.

Readings where the paper is silent:
  * a schedule is given as non-negative integer weights a_{i,l} (32-bit), one
    per response position, q_i(l) = a_{i,l} / A_i with A_i = sum_l a_{i,l}.
    Integer weights make the cut and the survival function exact: the cut is
    the first l whose running sum exceeds r, r = (u64 * A_i) >> 64 with u64
    built from two 32-bit words of one Philox block (stream 2, high word first);
    p_{i,t} = (sum_{l >= t} a_{i,l}) / A_i is one fp64 division of exact
    integers.  A rollout whose weights are all zero has no schedule: it is
    kept whole with p = 1;
  * Poisson sampling uses the URS stream (stream 0) with a per-token threshold
    floor(p_{i,t} * 2**32), so a constant p reproduces URS draw for draw;
  * weights with given probabilities: w = 1 / ((n_rollouts * T_i) * p_{i,t}),
    the integer product first, then one fp64 multiplication and one fp64
    division, then rounding to fp32;
  * prefix packing: rollout i of the truncated batch is its prompt (P_i
    tokens) followed by its first L_i response tokens; the row whose output
    scores response token t0 (0-based) is the row `shift` places before it
    (shift = 1: next-token prediction, needs P_i >= 1; shift = 0: the rows
    already are the scoring states).

Test infrastructure: not used by the product path.
"""
import math
import numpy as np

from .philox import philox4x32_10, philox4x32_10_array

STREAM_POISSON, STREAM_SCHEDULE = 0, 2


def _key(seed):
    seed = int(seed)
    return seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF


# ---------------------------------------------------------------- schedules

def schedule_total(a):
    """A_i = sum_l a_{i,l} as a Python integer."""
    return sum(int(x) for x in a)


def schedule_suffix(a):
    """[sum_{l >= t} a_l for t = 1..T] as Python integers (Eq. 8 times A_i)."""
    out, run = [0] * len(a), 0
    for j in range(len(a) - 1, -1, -1):
        run += int(a[j])
        out[j] = run
    return out


def schedule_cut_of(a, r):
    """First l (1-based) whose running sum a_1 + ... + a_l exceeds r, 0 <= r < A."""
    run = 0
    for j, x in enumerate(a):
        run += int(x)
        if run > r:
            return j + 1
    raise ValueError("r must be below the total weight")


def schedule_cut(a, seed, step, rollout_id):
    """L_i ~ q_i (Sec. 4, Eq. 7) by inversion of the integer running sum."""
    T = len(a)
    if T == 0:
        return 0
    A = schedule_total(a)
    if A == 0:
        return T
    words = philox4x32_10((0, rollout_id, STREAM_SCHEDULE, step), _key(seed))
    u64 = (words[0] << 32) | words[1]
    return schedule_cut_of(a, (u64 * A) >> 64)


def schedule_pi(a):
    """p_{i,t} = Pr(L_i >= t) for t = 1..T (Eq. 8) as fp64."""
    A = schedule_total(a)
    if A == 0:
        return np.ones(len(a), dtype=np.float64)
    return np.array([float(s) / float(A) for s in schedule_suffix(a)], dtype=np.float64)


def schedule_q(a):
    """q_i(l) for l = 1..T as fp64 (uniform on nothing: all mass on T when A = 0)."""
    A = schedule_total(a)
    if A == 0:
        q = np.zeros(len(a)); q[-1:] = 1.0
        return q
    return np.array([float(int(x)) / float(A) for x in a], dtype=np.float64)


def select_schedule(cu_seqlens, weights, seed=0, step=0, rollout_id_base=0, drop_zero_adv=None):
    """Cut every rollout of a packed batch by its own schedule.

    weights: [N] non-negative integers < 2**32 packed like the tokens.
    drop_zero_adv: optional [B] advantages (Eq. 2); a rollout whose advantage is
    exactly 0 keeps nothing (Eq. 3 with A = 0 gives S = 0 and a zero gradient at
    each of its tokens): its mask is cleared and its cut set to 0, while the
    survival function of every rollout, and so every weight, stays as it is.
    Returns dict(mask [N] bool, pi [N] fp64, cut_len [B] int32).
    """
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    B, N = len(cu) - 1, int(cu[-1])
    mask = np.zeros(N, dtype=bool)
    pi = np.zeros(N, dtype=np.float64)
    cut = np.zeros(B, dtype=np.int32)
    for i in range(B):
        lo, hi = int(cu[i]), int(cu[i + 1])
        a = [int(x) for x in weights[lo:hi]]
        L = schedule_cut(a, seed, step, rollout_id_base + i)
        if drop_zero_adv is not None and float(drop_zero_adv[i]) == 0.0:
            L = 0
        cut[i] = L
        mask[lo:lo + L] = True
        pi[lo:hi] = schedule_pi(a)
    return dict(mask=mask, pi=pi, cut_len=cut)


# ---------------------------------------------------------------- Poisson sampling

def poisson_threshold(p):
    """floor(p * 2**32) for one probability in [0, 1] (fp64 product, exact)."""
    p = float(p)
    if not (0.0 <= p <= 1.0):
        raise ValueError("probabilities must lie in [0,1]")
    return int(math.floor(p * 4294967296.0))


def poisson_mask(pi, seed, step, rollout_id):
    """m_t ~ Bernoulli(pi_t) independently for the T tokens of one rollout (Sec. 3.1)."""
    T = len(pi)
    if T == 0:
        return np.zeros(0, dtype=bool)
    t0 = np.arange(T, dtype=np.uint64)
    k0, k1 = _key(seed)
    words = philox4x32_10_array(t0 >> np.uint64(2), rollout_id, STREAM_POISSON, step, k0, k1)
    lane = (t0 & np.uint64(3)).astype(np.int64)
    u = np.choose(lane, [w.astype(np.uint64) for w in words])
    thr = np.array([poisson_threshold(p) for p in pi], dtype=np.uint64)
    return u < thr


def select_poisson(cu_seqlens, pi, seed=0, step=0, rollout_id_base=0, drop_zero_adv=None):
    """Independent Bernoulli(pi_n) mask for a packed batch; returns mask [N] bool.
    drop_zero_adv: as in select_schedule (zero-advantage rollouts keep nothing)."""
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    mask = np.zeros(int(cu[-1]), dtype=bool)
    for i in range(len(cu) - 1):
        lo, hi = int(cu[i]), int(cu[i + 1])
        if drop_zero_adv is not None and float(drop_zero_adv[i]) == 0.0:
            continue
        mask[lo:hi] = poisson_mask(np.asarray(pi[lo:hi], dtype=np.float64), seed, step, rollout_id_base + i)
    return mask


# ---------------------------------------------------------------- weights and compaction

def ht_weight_pi(T, pi_t, n_rollouts):
    """w = 1 / ((n_rollouts * T_i) * p_{i,t}) as float32 (Eq. 6 / Eq. 9 with Eq. 5's averaging)."""
    return np.float32(1.0 / (float(int(n_rollouts) * int(T)) * float(pi_t)))


def compact_pi(mask, pi, cu_seqlens, n_rollouts):
    """Stable compaction of the kept tokens with weights from given inclusion
    probabilities.  Same outputs as select.compact."""
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    B = len(cu) - 1
    kept_idx, kept_seq, kept_w = [], [], []
    cu_kept = np.zeros(B + 1, dtype=np.int32)
    for i in range(B):
        lo, hi = int(cu[i]), int(cu[i + 1])
        c = 0
        for n in range(lo, hi):
            if mask[n]:
                kept_idx.append(n)
                kept_seq.append(i)
                kept_w.append(ht_weight_pi(hi - lo, pi[n], n_rollouts))
                c += 1
        cu_kept[i + 1] = cu_kept[i] + c
    return dict(kept_idx=np.array(kept_idx, dtype=np.int32), kept_seq=np.array(kept_seq, dtype=np.int32),
                kept_w=np.array(kept_w, dtype=np.float32), cu_kept=cu_kept, n_kept=int(cu_kept[-1]))


# ---------------------------------------------------------------- prefix packing

def prefix_pack(prompt_len, cu_seqlens, cut_len, shift):
    """Truncated batch for a model body that runs only over kept prefixes (Sec. 4).

    The full packed input holds, per rollout, P_i prompt tokens then T_i
    response tokens.  Returns dict(
      cu_packed [B+1] int32   offsets of the truncated sequences (P_i + L_i rows each),
      src_idx   [M]   int32   row of the full packed input each truncated row comes from,
      position_ids [M] int32  0 .. P_i + L_i - 1 within each sequence,
      loss_row  [N_k] int32   truncated row whose output scores kept response token k
                              (kept tokens in ascending (i, t) order),
      total M, max_len  (longest truncated sequence)).
    """
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    B = len(cu) - 1
    P = np.zeros(B, dtype=np.int64) if prompt_len is None else np.asarray(prompt_len, dtype=np.int64)
    cu_packed = np.zeros(B + 1, dtype=np.int32)
    src_idx, position_ids, loss_row = [], [], []
    full_start, max_len = 0, 0
    for i in range(B):
        T, L = int(cu[i + 1] - cu[i]), int(cut_len[i])
        if not (0 <= L <= T):
            raise ValueError("cut outside [0, T]")
        if shift and L > 0 and P[i] < 1:
            raise ValueError("next-token shift needs at least one prompt token")
        rows = int(P[i]) + L
        for j in range(rows):
            src_idx.append(full_start + j)
            position_ids.append(j)
        for t0 in range(L):
            loss_row.append(int(cu_packed[i]) + int(P[i]) + t0 - shift)
        cu_packed[i + 1] = cu_packed[i] + rows
        max_len = max(max_len, rows)
        full_start += int(P[i]) + T
    return dict(cu_packed=cu_packed, src_idx=np.array(src_idx, dtype=np.int32),
                position_ids=np.array(position_ids, dtype=np.int32),
                loss_row=np.array(loss_row, dtype=np.int32), total=int(cu_packed[-1]), max_len=max_len)
