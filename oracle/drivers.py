"""Expectation drivers for the masked estimator (Prop. 1) and closed-form
variances (Sec. 3.1 second moment, Sec. 4 covariance, App. B.1 and B.4).

A "batch" is a dict: cu_seqlens [B+1], hidden [N, H], W [V, H], ids [N],
old_logp [N], adv [B]  (packed response tokens of B rollouts); optionally
ref_logp [N], beta_kl, kl_kind for the KL term of Eq. 4.

Test infrastructure: not used by the product path.
"""
import itertools
import numpy as np

from . import select as sel
from . import schedule as sch
from . import grpo


def _seq_of_token(cu):
    cu = np.asarray(cu, dtype=np.int64)
    return np.repeat(np.arange(len(cu) - 1), np.diff(cu))


def estimate(batch, mask, pi, eps_lo=0.2, eps_hi=0.2, n_rollouts=None):
    """Eq. 6 / Eq. 9 summed over the batch for an explicit mask and inclusion
    probabilities (no random numbers): weights m/(n_rollouts * T_i * p_{i,t}).

    Returns dict(loss, dH [N, H] with zero rows for dropped tokens, dW [V, H]).
    mask all True and pi all 1 gives the full-token GRPO objective of Eq. 5.
    """
    cu = np.asarray(batch["cu_seqlens"], dtype=np.int64)
    B = len(cu) - 1
    nB = B if n_rollouts is None else n_rollouts
    seq = _seq_of_token(cu)
    T = np.diff(cu)[seq].astype(np.float64)
    mask = np.asarray(mask, dtype=bool)
    kept = np.nonzero(mask)[0]
    w = 1.0 / (nB * T[kept] * np.asarray(pi, dtype=np.float64)[kept])
    out = grpo.loss_and_grads(np.asarray(batch["hidden"])[kept], batch["W"],
                              np.asarray(batch["ids"])[kept], np.asarray(batch["old_logp"])[kept],
                              np.asarray(batch["adv"], dtype=np.float64)[seq[kept]], w, eps_lo, eps_hi,
                              ref_logp=(np.asarray(batch["ref_logp"])[kept] if "ref_logp" in batch else None),
                              beta_kl=batch.get("beta_kl", 0.0), kl_kind=batch.get("kl_kind", grpo.KL_LOG_RATIO))
    dH = np.zeros(np.asarray(batch["hidden"]).shape, dtype=np.float64)
    dH[kept] = out["dH"]
    return dict(loss=out["loss"], dH=dH, dW=out["dW"])


def full_token(batch, eps_lo=0.2, eps_hi=0.2):
    """Full-token GRPO (Eq. 5): every token kept with probability one."""
    N = int(np.asarray(batch["cu_seqlens"])[-1])
    return estimate(batch, np.ones(N, bool), np.ones(N), eps_lo, eps_hi)


def _accumulate(acc, prob, est):
    for k in ("loss", "dH", "dW"):
        acc[k] = acc.get(k, 0.0) + prob * est[k]
    acc["loss_sq"] = acc.get("loss_sq", 0.0) + prob * est["loss"] ** 2
    acc["prob"] = acc.get("prob", 0.0) + prob


def enumerate_urs(batch, p, eps_lo=0.2, eps_hi=0.2):
    """Exact expectation over all 2**N independent Bernoulli(p) masks."""
    N = int(np.asarray(batch["cu_seqlens"])[-1])
    pi = np.full(N, float(p))
    acc = {}
    for bits in itertools.product((False, True), repeat=N):
        m = np.array(bits, dtype=bool)
        k = int(m.sum())
        prob = (p ** k) * ((1.0 - p) ** (N - k))
        if prob == 0.0:
            continue
        _accumulate(acc, prob, estimate(batch, m, pi, eps_lo, eps_hi))
    return acc


def enumerate_rpc(batch, C=1, eps_lo=0.2, eps_hi=0.2):
    """Exact expectation over every combination of uniform cut points L_i in
    {C_i..T_i}, each rollout independent."""
    cu = np.asarray(batch["cu_seqlens"], dtype=np.int64)
    Ts = np.diff(cu)
    pi = np.concatenate([sel.inclusion_prob(sel.RPC, int(T), C=C) for T in Ts])
    ranges = [range(sel.rpc_min_cut(int(T), C), int(T) + 1) for T in Ts]
    acc = {}
    for cuts in itertools.product(*ranges):
        prob = 1.0
        m = np.zeros(int(cu[-1]), dtype=bool)
        for i, L in enumerate(cuts):
            prob /= len(ranges[i])
            m[cu[i]:cu[i] + L] = True
        _accumulate(acc, prob, estimate(batch, m, pi, eps_lo, eps_hi))
    return acc


def enumerate_schedule(batch, weights, eps_lo=0.2, eps_hi=0.2):
    """Exact expectation over every combination of cuts L_i ~ q_i, q_i given by
    integer weights per response position (Sec. 4, Eq. 7-9), rollouts independent."""
    cu = np.asarray(batch["cu_seqlens"], dtype=np.int64)
    per = [[int(x) for x in weights[cu[i]:cu[i + 1]]] for i in range(len(cu) - 1)]
    pi = np.concatenate([sch.schedule_pi(a) for a in per])
    qs = [sch.schedule_q(a) for a in per]
    acc = {}
    for cuts in itertools.product(*[range(1, len(a) + 1) for a in per]):
        prob = 1.0
        m = np.zeros(int(cu[-1]), dtype=bool)
        for i, L in enumerate(cuts):
            prob *= qs[i][L - 1]
            m[cu[i]:cu[i] + L] = True
        if prob == 0.0:
            continue
        _accumulate(acc, prob, estimate(batch, m, pi, eps_lo, eps_hi))
    return acc


def enumerate_poisson(batch, pi, eps_lo=0.2, eps_hi=0.2):
    """Exact expectation over all 2**N independent masks m_n ~ Bernoulli(pi_n) (Sec. 3.1)."""
    pi = np.asarray(pi, dtype=np.float64)
    N = len(pi)
    acc = {}
    for bits in itertools.product((False, True), repeat=N):
        m = np.array(bits, dtype=bool)
        prob = float(np.prod(np.where(m, pi, 1.0 - pi)))
        if prob == 0.0:
            continue
        _accumulate(acc, prob, estimate(batch, m, pi, eps_lo, eps_hi))
    return acc


def det_trunc(batch, beta, eps_lo=0.2, eps_hi=0.2):
    """The single deterministic-truncation estimate (weight 1 on the prefix)."""
    cu = np.asarray(batch["cu_seqlens"], dtype=np.int64)
    m = np.zeros(int(cu[-1]), dtype=bool)
    for i in range(len(cu) - 1):
        m[cu[i]:cu[i] + sel.det_keep(int(cu[i + 1] - cu[i]), beta)] = True
    return estimate(batch, m, np.ones(len(m)), eps_lo, eps_hi)


def monte_carlo(batch, scheme, seeds, p=1.0, C=1, beta=1.0, eps_lo=0.2, eps_hi=0.2, step=0):
    """Mean and mean-of-squares of the estimate over seeded draws of select()."""
    acc = {}
    for s in seeds:
        d = sel.select(batch["cu_seqlens"], scheme, p=p, C=C, beta=beta, seed=s, step=step)
        pi = np.where(d["pi"] > 0, d["pi"], 1.0)
        _accumulate(acc, 1.0 / len(seeds), estimate(batch, d["mask"], pi, eps_lo, eps_hi))
    return acc


# ---- closed forms for one rollout with per-token losses Lt (t = 1..T) ----

def ht_value(Lt, mask, pi):
    """mu_hat = (1/T) sum_t m_t L_t / p_t   (Eq. 6)."""
    Lt = np.asarray(Lt, dtype=np.float64)
    m = np.asarray(mask, dtype=bool)
    return float(np.sum(Lt[m] / np.asarray(pi, dtype=np.float64)[m]) / len(Lt))


def var_independent(Lt, pi):
    """App. B.4: (1/T^2) sum_t L_t^2 (1 - p_t)/p_t for independent masks."""
    Lt = np.asarray(Lt, dtype=np.float64)
    pi = np.asarray(pi, dtype=np.float64)
    return float(np.sum(Lt ** 2 * (1.0 - pi) / pi) / len(Lt) ** 2)


def var_rpc_stopping(Lt, pi, q):
    """App. B.1: (1/T^2) (E[(sum_{t<=tau} L_t/p_t)^2] - (sum_t L_t)^2) with
    Pr(tau = l) = q[l-1]."""
    Lt = np.asarray(Lt, dtype=np.float64)
    partial = np.cumsum(Lt / np.asarray(pi, dtype=np.float64))
    second = float(np.sum(np.asarray(q, dtype=np.float64) * partial ** 2))
    return (second - float(Lt.sum()) ** 2) / len(Lt) ** 2
