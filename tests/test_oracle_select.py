"""Pins for oracle.select against what the paper fixes: Sec. 3.1 (URS), Sec. 4
(RPC survival function Eq. 8, uniform and minimum-cutoff closed forms, mask
covariance, deterministic truncation), App. B.2 (selected-token ratio)."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import select as sel


# ---------------------------------------------------------------- URS ----

def test_urs_threshold_exact_cases():
    assert sel.urs_threshold(1.0) == 2 ** 32
    assert sel.urs_threshold(0.5) == 2 ** 31
    assert sel.urs_threshold(0.25) == 2 ** 30
    with pytest.raises(ValueError):
        sel.urs_threshold(0.0)
    with pytest.raises(ValueError):
        sel.urs_threshold(1.5)


def test_urs_p1_keeps_every_token():
    for T in (1, 3, 64, 1000):
        assert sel.urs_mask(T, 1.0, seed=11, step=3, rollout_id=5).all()


@pytest.mark.parametrize("p", [0.25, 0.5, 0.8])
def test_urs_keep_rate_binomial(p):
    # Sec. 3.1: m ~ Bernoulli(p) i.i.d.  4e6 draws, 5-sigma band
    n = 0
    k = 0
    for gid in range(4):
        m = sel.urs_mask(1_000_000, p, seed=2024, step=1, rollout_id=gid)
        n += m.size
        k += int(m.sum())
    sigma = math.sqrt(n * p * (1 - p))
    assert abs(k - n * p) < 5 * sigma


def test_urs_independence_between_neighbours():
    # lag-1 correlation of i.i.d. Bernoulli draws is ~ N(0, 1/n)
    m = sel.urs_mask(1_000_000, 0.5, seed=7, step=0, rollout_id=0).astype(np.float64)
    c = np.corrcoef(m[:-1], m[1:])[0, 1]
    assert abs(c) < 5e-3


def test_urs_depends_only_on_seed_step_rollout_and_position():
    a = sel.urs_mask(100, 0.5, seed=3, step=4, rollout_id=9)
    b = sel.urs_mask(60, 0.5, seed=3, step=4, rollout_id=9)
    assert (a[:60] == b).all()
    assert not (a == sel.urs_mask(100, 0.5, seed=3, step=5, rollout_id=9)).all()
    assert not (a == sel.urs_mask(100, 0.5, seed=3, step=4, rollout_id=8)).all()
    assert not (a == sel.urs_mask(100, 0.5, seed=4, step=4, rollout_id=9)).all()
    # batch offset invariance: rollout_id_base shifts the global id
    cu = [0, 10, 25]
    s1 = sel.select(cu, sel.URS, p=0.5, seed=3, step=4, rollout_id_base=8)
    assert (s1["mask"][10:25] == a[:15]).all()


# ---------------------------------------------------------------- RPC ----

def _closed_form_rows(golden_dir):
    for line in open(os.path.join(golden_dir, "rpc_closed_forms.txt")):
        if line.startswith("#") or not line.strip():
            continue
        head, el, probs = [x.strip() for x in line.split("|")]
        T, C = [int(x) for x in head.split()]
        yield T, C, Fraction(el), [Fraction(x) for x in probs.split()]


def test_rpc_inclusion_prob_matches_printed_closed_forms(golden_dir):
    rows = list(_closed_form_rows(golden_dir))
    assert len(rows) == 6
    for T, C, EL, probs in rows:
        pi = sel.inclusion_prob(sel.RPC, T, C=C)
        assert np.allclose(pi, [float(x) for x in probs], rtol=0, atol=1e-15)
        # E[L] = sum_t p_t (Sec. 4)
        assert abs(pi.sum() - float(EL)) < 1e-12


@pytest.mark.parametrize("T,C", [(1, 1), (2, 1), (17, 1), (17, 5), (100, 100), (9, 30)])
def test_rpc_survival_properties(T, C):
    # Eq. 8: p_1 = 1, non-increasing, p_T = q(T) = 1/n > 0
    pi = sel.inclusion_prob(sel.RPC, T, C=C)
    n = T - min(max(C, 1), T) + 1
    assert pi[0] == 1.0
    assert (np.diff(pi) <= 0).all()
    assert abs(pi[-1] - 1.0 / n) < 1e-15
    # survival function of the uniform law: p_t = sum_{l >= t} q(l)
    Ci = T - n + 1
    q = np.array([1.0 / n if l >= Ci else 0.0 for l in range(1, T + 1)])
    assert np.allclose(pi, q[::-1].cumsum()[::-1], atol=1e-15)
    # expected retained length (C+T)/2 and ratio 1/2 + C/(2T)  (App. B.2)
    assert abs(pi.sum() - (Ci + T) / 2) < 1e-12
    assert abs(pi.sum() / T - (0.5 + Ci / (2 * T))) < 1e-12


@pytest.mark.parametrize("T,C", [(12, 1), (12, 4), (5, 9)])
def test_rpc_cut_range_uniformity_and_mean(T, C):
    K = 30000
    Ls = np.array([sel.rpc_cut(T, C, seed=99, step=0, rollout_id=g) for g in range(K)])
    Ci = min(max(C, 1), T)
    n = T - Ci + 1
    assert Ls.min() >= Ci and Ls.max() <= T
    if n == 1:
        assert (Ls == T).all()
        return
    counts = np.bincount(Ls, minlength=T + 1)[Ci:]
    chi2 = ((counts - K / n) ** 2 / (K / n)).sum()
    # chi-square with n-1 dof: mean n-1, std sqrt(2(n-1)); 6-sigma band
    assert chi2 < (n - 1) + 6 * math.sqrt(2 * (n - 1))
    sd = math.sqrt((n * n - 1) / 12.0 / K)
    assert abs(Ls.mean() - (Ci + T) / 2) < 5 * sd


def test_rpc_mask_frequency_matches_inclusion_prob():
    # ties the drawn mask to the p_{i,t} used in the weights (Eq. 7-8)
    T, C, K = 9, 3, 40000
    cu = [0, T]
    freq = np.zeros(T)
    for s in range(K):
        freq += sel.select(cu, sel.RPC, C=C, seed=s, step=2)["mask"]
    freq /= K
    pi = sel.inclusion_prob(sel.RPC, T, C=C)
    sd = np.sqrt(np.maximum(pi * (1 - pi), 1e-12) / K)
    assert (np.abs(freq - pi) <= 5 * sd + 1e-12).all()


def test_rpc_mask_covariance_closed_form():
    # Sec. 4: Cov(m_s, m_t) = p_t (1 - p_s) for s <= t, by enumerating the cuts
    T, C = 8, 2
    pi = sel.inclusion_prob(sel.RPC, T, C=C)
    cuts = range(sel.rpc_min_cut(T, C), T + 1)
    M = np.array([[1.0 if t <= L else 0.0 for t in range(1, T + 1)] for L in cuts])
    cov = (M.T @ M) / len(cuts) - np.outer(M.mean(0), M.mean(0))
    for s in range(T):
        for t in range(s, T):
            assert abs(cov[s, t] - pi[t] * (1 - pi[s])) < 1e-14
    assert np.allclose(M.mean(0), pi, atol=1e-15)


def test_rpc_always_keeps_first_token_and_prefix_shape():
    cu = np.concatenate([[0], np.cumsum([1, 2, 7, 30, 1, 64, 65])])
    for seed in range(50):
        d = sel.select(cu, sel.RPC, C=1, seed=seed)
        for i in range(len(cu) - 1):
            m = d["mask"][cu[i]:cu[i + 1]]
            L = d["cut_len"][i]
            assert 1 <= L <= len(m)
            assert m[:L].all() and not m[L:].any()


# ------------------------------------------------------- DET, weights ----

def test_det_trunc_floor_rule():
    assert sel.det_keep(1, 0.5) == 0          # literal floor: a length-1 rollout keeps nothing
    assert sel.det_keep(7, 0.5) == 3
    assert sel.det_keep(8, 0.5) == 4
    assert sel.det_keep(10, 1.0) == 10
    pi = sel.inclusion_prob(sel.DET, 7, beta=0.5)
    assert pi.tolist() == [1, 1, 1, 0, 0, 0, 0]


def test_ht_weight_closed_forms():
    B = 6
    # RPC with C=1: w = 1/(B (T-t+1))
    for T in (1, 5, 33):
        for t in range(1, T + 1):
            w = sel.ht_weight(sel.RPC, T, t, B, C=1)
            assert w == np.float32(1.0 / (B * (T - t + 1)))
    # URS: 1/(B T p);  FULL / DET: 1/(B T)
    assert sel.ht_weight(sel.URS, 10, 3, B, p=0.5) == np.float32(1.0 / 30.0)
    assert sel.ht_weight(sel.FULL, 10, 3, B) == np.float32(1.0 / 60.0)
    assert sel.ht_weight(sel.DET, 10, 3, B) == np.float32(1.0 / 60.0)


@pytest.mark.parametrize("scheme,kw", [(sel.URS, dict(p=0.3)), (sel.RPC, dict(C=1)), (sel.RPC, dict(C=4)),
                                       (sel.FULL, {})])
def test_ht_weight_is_reciprocal_of_B_T_pi(scheme, kw):
    B, T = 5, 11
    pi = sel.inclusion_prob(scheme, T, **kw)
    for t in range(1, T + 1):
        w = float(sel.ht_weight(scheme, T, t, B, **kw))
        assert abs(w * (B * T * pi[t - 1]) - 1.0) < 2e-7     # fp32 rounding only
    ws = sel.ht_weights_rollout(scheme, T, np.arange(1, T + 1), B, **kw)
    assert all(ws[t - 1] == sel.ht_weight(scheme, T, t, B, **kw) for t in range(1, T + 1))


def test_sum_of_weights_has_expectation_one_over_B():
    # E[ sum_t m_t w_t ] = (1/B) * (1/T) sum_t p_t / p_t = 1/B   (Eq. 6 with L = 1)
    T, B, C = 7, 3, 2
    cuts = range(sel.rpc_min_cut(T, C), T + 1)
    tot = 0.0
    for L in cuts:
        tot += sum(float(sel.ht_weight(sel.RPC, T, t, B, C=C)) for t in range(1, L + 1)) / len(cuts)
    assert abs(tot - 1.0 / B) < 1e-7


# ---------------------------------------------------------- compaction ----

def test_compact_against_brute_force_and_mixed_schemes():
    rng = np.random.default_rng(0)
    T = np.array([1, 70, 0, 33, 64, 5, 128, 2])
    cu = np.concatenate([[0], np.cumsum(T)])
    schemes = np.array([sel.URS, sel.DET, sel.URS, sel.RPC, sel.FULL, sel.DET, sel.URS, sel.RPC])
    d = sel.select(cu, sel.URS, p=0.5, C=3, beta=0.5, seed=42, step=1, scheme_per_rollout=schemes)
    c = sel.compact(d["mask"], cu, 8, sel.URS, p=0.5, C=3, scheme_per_rollout=schemes)
    idx, seq, w = [], [], []
    for i in range(len(T)):
        for t0 in range(T[i]):
            if d["mask"][cu[i] + t0]:
                idx.append(cu[i] + t0)
                seq.append(i)
                w.append(sel.ht_weight(int(schemes[i]), int(T[i]), t0 + 1, 8, p=0.5, C=3))
    assert c["kept_idx"].tolist() == idx
    assert c["kept_seq"].tolist() == seq
    assert c["kept_w"].tolist() == [float(x) for x in w]
    assert c["n_kept"] == len(idx) == int(d["mask"].sum())
    assert (np.diff(c["kept_idx"]) > 0).all()
    for i in range(len(T)):
        assert c["cu_kept"][i + 1] - c["cu_kept"][i] == d["mask"][cu[i]:cu[i + 1]].sum()
    # cut_len bookkeeping
    assert d["cut_len"][1] == 35 and d["cut_len"][5] == 2 and d["cut_len"][4] == 64 and d["cut_len"][2] == 0


def test_pack_mask_bits_roundtrip():
    rng = np.random.default_rng(1)
    for N in (0, 1, 31, 32, 33, 64, 65, 1000):
        m = rng.random(N) < 0.5
        words = sel.pack_mask_bits(m)
        assert words.dtype == np.uint32 and len(words) == 2 * ((N + 63) // 64)
        for n in range(N):
            assert bool((int(words[n >> 5]) >> (n & 31)) & 1) == bool(m[n])
        assert sum(bin(int(x)).count("1") for x in words) == int(m.sum())


def test_full_scheme_and_empty_batch():
    d = sel.select([0, 4, 4, 9], sel.FULL)
    assert d["mask"].all() and (d["pi"] == 1).all() and d["cut_len"].tolist() == [4, 0, 5]
    c = sel.compact(d["mask"], [0, 4, 4, 9], 3, sel.FULL)
    assert c["kept_idx"].tolist() == list(range(9)) and c["cu_kept"].tolist() == [0, 4, 4, 9]
    d0 = sel.select([0, 0], sel.URS, p=0.5)
    assert d0["mask"].size == 0


# ------------------------------------------------- zero-advantage rollouts ----

def test_dropping_zero_advantage_rollouts_leaves_the_estimate_unchanged():
    # Eq. 3 with A = 0: S = 0 and dS/dlogp = 0 at every token of the rollout, whatever the ratio
    from oracle import drivers, grpo
    from test_oracle_grpo import tiny_batch
    b = tiny_batch(51, [5, 4, 6, 3])
    b["adv"] = np.array([0.7, 0.0, -1.2, 0.0])
    cu = b["cu_seqlens"]
    for scheme, kw in ((sel.FULL, {}), (sel.URS, dict(p=0.5)), (sel.RPC, dict(C=2))):
        keep_all = sel.select(cu, scheme, seed=4, **kw)
        dropped = sel.select(cu, scheme, seed=4, drop_zero_adv=b["adv"], **kw)
        assert not dropped["mask"][cu[1]:cu[2]].any() and not dropped["mask"][cu[3]:cu[4]].any()
        assert dropped["cut_len"][1] == 0 and dropped["cut_len"][3] == 0
        for i in (0, 2):                                       # the other rollouts draw exactly as before
            assert np.array_equal(dropped["mask"][cu[i]:cu[i + 1]], keep_all["mask"][cu[i]:cu[i + 1]])
        assert np.array_equal(dropped["pi"], keep_all["pi"])
        e1 = drivers.estimate(b, keep_all["mask"], keep_all["pi"])
        e2 = drivers.estimate(b, dropped["mask"], dropped["pi"])
        assert e1["loss"] == e2["loss"] or abs(e1["loss"] - e2["loss"]) < 1e-15
        assert np.abs(e1["dW"] - e2["dW"]).max() < 1e-15 and np.abs(e1["dH"] - e2["dH"]).max() < 1e-15
    # with a KL term the dropped tokens would have contributed: the shortcut is exact only for beta_KL = 0
    bk = dict(b, ref_logp=b["old_logp"] + 0.3, beta_kl=0.5, kl_kind=grpo.KL_NONNEG)
    e1 = drivers.estimate(bk, keep_all["mask"], keep_all["pi"])
    e2 = drivers.estimate(bk, dropped["mask"], dropped["pi"])
    assert abs(e1["loss"] - e2["loss"]) > 1e-4


def test_equal_rewards_give_exactly_zero_advantage_and_the_group_is_dropped():
    from oracle import grpo
    A = grpo.advantages(np.array([[1.0, 1.0, 1.0, 1.0], [0.0, 1.0, 0.0, 1.0], [0.0, 0.0, 0.0, 0.0]])).reshape(-1)
    assert (A[:4] == 0).all() and (A[8:] == 0).all() and (A[4:8] != 0).all()
    cu = np.arange(13) * 10
    d = sel.select(cu, sel.FULL, drop_zero_adv=A)
    assert d["mask"].sum() == 40 and d["mask"][40:80].all()
