"""Token selection, inclusion probabilities, Horvitz-Thompson weights, compaction.

Follows Sec. 3.1 (random masking m_{i,t} ~ Bernoulli(p_{i,t}); URS with
constant p), Sec. 4 (RPC: cut L_i, mask 1{t <= L_i}, survival p_{i,t} =
Pr(L_i >= t), Eq. 7-8; uniform cutoff; minimum-cutoff variant with C;
deterministic truncation K_i = floor(beta T_i)) and the estimator of Eq. 6 /
Eq. 9 combined with the 1/G * 1/|o_i| averaging of Eq. 5.

Token positions t are 1-based in the paper; arrays here are indexed by
t0 = t - 1.  Rollouts are packed back to back: token (i, t0) sits at packed
position cu_seqlens[i] + t0.

Readings where the paper is silent (also listed in the design notes):
  * random bits: Philox4x32-10, key = (seed low word, seed high word),
    counter = (t0 >> 2, global rollout id, stream, step); stream 0 feeds the
    URS token draws (word t0 & 3 of the block), stream 1 the RPC cut (word 0);
  * Bernoulli(p): keep iff u32 < floor(p * 2**32)  (p = 1 keeps everything);
  * uniform integer on n values: (u32 * n) >> 32;
  * C > T_i is clamped to T_i (then L_i = T_i);  L_i >= 1 always.

Test infrastructure: not used by the product path.
"""
import math
import numpy as np

from .philox import philox4x32_10, philox4x32_10_array

FULL, URS, RPC, DET = 0, 1, 2, 3
STREAM_URS, STREAM_RPC = 0, 1


def _key(seed):
    seed = int(seed)
    return seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF


def urs_threshold(p):
    """Integer threshold for Bernoulli(p) on a 32-bit word (p in (0,1])."""
    if not (0.0 < p <= 1.0):
        raise ValueError("p must be in (0,1]")
    return int(math.floor(p * 4294967296.0))


def urs_mask(T, p, seed, step, rollout_id):
    """m_{i,t} ~ Bernoulli(p) independently for t = 1..T  (Sec. 3.1, URS)."""
    t0 = np.arange(T, dtype=np.uint64)
    k0, k1 = _key(seed)
    words = philox4x32_10_array(t0 >> np.uint64(2), rollout_id, STREAM_URS, step, k0, k1)
    lane = (t0 & np.uint64(3)).astype(np.int64)
    u = np.choose(lane, [w.astype(np.uint64) for w in words]) if T > 0 else np.zeros(0, np.uint64)
    return u < np.uint64(urs_threshold(p))


def rpc_min_cut(T, C):
    """C_i = min(max(C, 1), T_i): first position that may be the cut."""
    return min(max(int(C), 1), int(T))


def rpc_cut(T, C, seed, step, rollout_id):
    """L_i ~ Uniform{C_i, ..., T_i}  (Sec. 4, uniform and minimum-cutoff RPC)."""
    if T <= 0:
        return 0
    Ci = rpc_min_cut(T, C)
    n = T - Ci + 1
    k0, k1 = _key(seed)
    u = philox4x32_10((0, rollout_id, STREAM_RPC, step), (k0, k1))[0]
    return Ci + ((u * n) >> 32)


def det_keep(T, beta):
    """K_i = floor(beta * T_i)  (Sec. 4, deterministic truncation)."""
    if not (0.0 < beta <= 1.0):
        raise ValueError("beta must be in (0,1]")
    return int(math.floor(float(beta) * float(T)))


def inclusion_prob(scheme, T, p=1.0, C=1, beta=1.0):
    """p_{i,t} for t = 1..T as an fp64 array.

    FULL: 1.  URS: p.  RPC: 1 for t <= C_i, (T-t+1)/(T-C_i+1) after (Eq. 8 with
    q uniform on {C_i..T}).  DET: 1 for t <= K, 0 after (violates p > 0; the
    biased control of Sec. 4).
    """
    t = np.arange(1, T + 1, dtype=np.float64)
    if scheme == FULL:
        return np.ones(T)
    if scheme == URS:
        return np.full(T, float(p))
    if scheme == RPC:
        Ci = rpc_min_cut(T, C) if T > 0 else 1
        n = T - Ci + 1
        return np.where(t <= Ci, 1.0, (T - t + 1.0) / n)
    if scheme == DET:
        return (t <= det_keep(T, beta)).astype(np.float64)
    raise ValueError("unknown scheme")


def ht_weight(scheme, T, t, n_rollouts, p=1.0, C=1):
    """w_{i,t} = 1 / (n_rollouts * T_i * p_{i,t}) for a KEPT token, as float32.

    This is the factor multiplying S_{i,t} in the batch estimate: 1/G and
    1/|o_i| of Eq. 5, the mean over prompts (n_rollouts = P*G), and
    m_{i,t}/p_{i,t} of Eq. 6.  Evaluated as one fp64 division, then rounded to
    fp32.  DET uses p := 1 on its kept prefix.
    """
    Bn = float(n_rollouts)
    T = int(T)
    t = int(t)
    if scheme == URS:
        w = 1.0 / (Bn * float(T) * float(p))
    elif scheme == RPC and t > rpc_min_cut(T, C):
        n = T - rpc_min_cut(T, C) + 1
        w = float(n) / (float(T - t + 1) * float(T) * Bn)
    else:
        w = 1.0 / (Bn * float(T))
    return np.float32(w)


def select(cu_seqlens, scheme, p=1.0, C=1, beta=1.0, seed=0, step=0,
           rollout_id_base=0, scheme_per_rollout=None, drop_zero_adv=None):
    """Draw the mask for a packed batch.

    Returns dict(mask [N] bool, pi [N] fp64, cut_len [B] int32) where cut_len
    is L_i (RPC), K_i (DET) or T_i (FULL, URS).

    drop_zero_adv: optional [B] advantages (Eq. 2).  A rollout whose advantage
    is exactly 0 has S_{i,t} = 0 and zero gradient at every token (Eq. 3 with
    A = 0), so when the token loss has no KL term it can be left out without
    changing the estimate: its mask is cleared and its cut_len set to 0.  The
    inclusion probabilities (and so the weights of the other rollouts) stay as
    they are.
    """
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    B = len(cu) - 1
    N = int(cu[-1])
    mask = np.zeros(N, dtype=bool)
    pi = np.zeros(N, dtype=np.float64)
    cut = np.zeros(B, dtype=np.int32)
    for i in range(B):
        T = int(cu[i + 1] - cu[i])
        s = int(scheme_per_rollout[i]) if scheme_per_rollout is not None else scheme
        gid = rollout_id_base + i
        sl = slice(int(cu[i]), int(cu[i + 1]))
        pi[sl] = inclusion_prob(s, T, p, C, beta)
        if s == FULL:
            mask[sl] = True
            cut[i] = T
        elif s == URS:
            mask[sl] = urs_mask(T, p, seed, step, gid)
            cut[i] = T
        elif s == RPC:
            L = rpc_cut(T, C, seed, step, gid)
            mask[sl] = np.arange(1, T + 1) <= L
            cut[i] = L
        elif s == DET:
            K = det_keep(T, beta)
            mask[sl] = np.arange(1, T + 1) <= K
            cut[i] = K
        else:
            raise ValueError("unknown scheme")
        if drop_zero_adv is not None and float(drop_zero_adv[i]) == 0.0:
            mask[sl] = False
            cut[i] = 0
    return dict(mask=mask, pi=pi, cut_len=cut)


def pack_mask_bits(mask):
    """Mask as little-endian bit words: bit (n & 31) of word n >> 5 is m_n.
    Length 2*ceil(N/64) uint32 words (whole 64-token groups)."""
    N = len(mask)
    nwords = 2 * ((N + 63) // 64)
    bits = np.zeros(nwords * 32, dtype=np.uint8)
    bits[:N] = mask
    return np.packbits(bits.reshape(-1, 32), axis=1, bitorder="little").view(np.uint32).reshape(-1)


def ht_weights_rollout(scheme, T, t, n_rollouts, p=1.0, C=1):
    """ht_weight for an array t of kept 1-based positions of one rollout (same
    single fp64 division per token, then fp32)."""
    Bn = float(n_rollouts)
    t = np.asarray(t, dtype=np.float64)
    base = np.full(t.shape, 1.0 / (Bn * float(T)))
    if scheme == URS:
        w = np.full(t.shape, 1.0 / (Bn * float(T) * float(p)))
    elif scheme == RPC:
        Ci = rpc_min_cut(T, C)
        n = T - Ci + 1
        w = np.where(t > Ci, float(n) / ((float(T) - t + 1.0) * float(T) * Bn), base)
    else:
        w = base
    return w.astype(np.float32)


def compact(mask, cu_seqlens, n_rollouts, scheme, p=1.0, C=1, scheme_per_rollout=None):
    """Stable mask -> index compaction with per-kept-token HT weights.

    Kept tokens are listed in ascending (i, t) order.  Returns dict(kept_idx
    [N_k] int32 packed positions, kept_seq [N_k] int32 rollout index, kept_w
    [N_k] float32, cu_kept [B+1] int32, n_kept int).
    """
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    B = len(cu) - 1
    kept_idx, kept_seq, kept_w = [], [], []
    cu_kept = np.zeros(B + 1, dtype=np.int32)
    for i in range(B):
        T = int(cu[i + 1] - cu[i])
        s = int(scheme_per_rollout[i]) if scheme_per_rollout is not None else scheme
        t0 = np.nonzero(mask[int(cu[i]):int(cu[i + 1])])[0]
        if len(t0) == 0:          # nothing kept (also T_i = 0): no weights to form
            cu_kept[i + 1] = cu_kept[i]
            continue
        kept_idx.append(cu[i] + t0)
        kept_seq.append(np.full(len(t0), i))
        kept_w.append(ht_weights_rollout(s, T, t0 + 1, n_rollouts, p, C))
        cu_kept[i + 1] = cu_kept[i] + len(t0)
    cat = lambda xs, dt: (np.concatenate(xs).astype(dt) if xs else np.zeros(0, dt))
    return dict(kept_idx=cat(kept_idx, np.int32), kept_seq=cat(kept_seq, np.int32),
                kept_w=cat(kept_w, np.float32), cu_kept=cu_kept, n_kept=int(cu_kept[-1]))
