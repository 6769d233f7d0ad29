"""Pins for oracle.schedule: general cut-length distributions (Sec. 4, Eq. 7-9:
survival function, its stated properties, the uniform and minimum-cutoff closed
forms, Prop. 1 and App. B.1 by enumeration), Poisson sampling with
token-dependent probabilities (Sec. 3.1, Eq. 6, App. B.4), prefix packing."""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import drivers, grpo, schedule as sch
from oracle import select as sel
from test_oracle_grpo import tiny_batch, _token_losses


# ---------------------------------------------------------------- survival function (Eq. 8)

def test_survival_uniform_schedule_matches_printed_closed_form():
    # q(l) = 1/T  =>  p_t = (T - t + 1)/T,  sum_t p_t = E[L] = (T + 1)/2
    for T in (1, 2, 7, 100):
        pi = sch.schedule_pi([1] * T)
        assert np.array_equal(pi, np.array([(T - t + 1) / T for t in range(1, T + 1)]))
        assert np.isclose(pi.sum(), (T + 1) / 2, rtol=1e-14)
        # any common scale of the integer weights is the same distribution
        assert np.array_equal(sch.schedule_pi([12345] * T), pi)


@pytest.mark.parametrize("T,C", [(9, 4), (20, 1), (5, 5), (3000, 100)])
def test_survival_minimum_cutoff_schedule_matches_printed_closed_form(T, C):
    # weights 0 below C, 1 on C..T  =>  p_t = 1 (t <= C), (T-t+1)/(T-C+1) after; E[L] = (C+T)/2
    a = [0] * (C - 1) + [1] * (T - C + 1)
    pi = sch.schedule_pi(a)
    assert np.array_equal(pi, sel.inclusion_prob(sel.RPC, T, C=C))
    assert np.isclose(pi.sum(), (C + T) / 2, rtol=1e-13)


def test_survival_properties_for_arbitrary_weights():
    rng = np.random.default_rng(5)
    for T in (1, 2, 13, 200):
        a = rng.integers(0, 2 ** 32, T).tolist()
        a[-1] = max(a[-1], 1)                                  # q(T) > 0 as the paper requires
        pi = sch.schedule_pi(a)
        A = sum(a)
        assert pi[0] == 1.0                                    # p_1 = 1
        assert (np.diff(pi) <= 0).all()                        # non-increasing
        assert pi[-1] == a[-1] / A and pi[-1] > 0              # p_T = q(T) > 0
        # against exact rationals, and sum_t p_t = E[L]
        exact = [Fraction(sum(a[t:]), A) for t in range(T)]
        assert all(abs(Fraction(float(x)) - e) <= Fraction(1, 2 ** 52) for x, e in zip(pi, exact))
        EL = sum(Fraction(x, A) * (l + 1) for l, x in enumerate(a))
        assert abs(Fraction(float(pi.sum())) - EL) < Fraction(T, 2 ** 48)


def test_weights_are_full_32_bit_and_sums_do_not_wrap():
    a = [2 ** 32 - 1] * 40000                                  # total ~ 2^47.3
    pi = sch.schedule_pi(a)
    assert pi[0] == 1.0 and pi[-1] == 1 / 40000 and sch.schedule_total(a) == 40000 * (2 ** 32 - 1)


def test_zero_weight_rollout_is_kept_whole():
    assert sch.schedule_cut([0, 0, 0], 1, 2, 3) == 3
    assert np.array_equal(sch.schedule_pi([0, 0, 0]), np.ones(3))
    assert sch.schedule_cut([], 1, 2, 3) == 0


# ---------------------------------------------------------------- the cut (Eq. 7)

def test_inversion_assigns_exactly_a_l_values_of_r_to_each_cut():
    a = [3, 0, 5, 1, 0, 2]
    counts = [0] * len(a)
    for r in range(sum(a)):
        counts[sch.schedule_cut_of(a, r) - 1] += 1
    assert counts == a
    with pytest.raises(ValueError):
        sch.schedule_cut_of(a, sum(a))


def test_cut_never_lands_on_zero_weight_and_follows_q():
    a = [0, 4, 0, 1, 3, 0, 2]                                  # A = 10
    n = 20000
    hist = np.zeros(len(a))
    for gid in range(n):
        L = sch.schedule_cut(a, seed=99, step=0, rollout_id=gid)
        hist[L - 1] += 1
    assert hist[[0, 2, 5]].sum() == 0
    q = sch.schedule_q(a)
    nz = q > 0
    chi2 = float(((hist[nz] - n * q[nz]) ** 2 / (n * q[nz])).sum())
    assert chi2 < 18.5                                          # 3 dof, p ~ 3e-4


def test_uniform_schedule_cut_has_mean_T_plus_1_over_2():
    T, n = 101, 20000
    Ls = np.array([sch.schedule_cut([7] * T, seed=5, step=1, rollout_id=g) for g in range(n)])
    assert Ls.min() >= 1 and Ls.max() <= T
    sigma = math.sqrt((T * T - 1) / 12 / n)
    assert abs(Ls.mean() - (T + 1) / 2) < 5 * sigma


def test_cut_depends_only_on_seed_step_and_global_rollout_id():
    rng = np.random.default_rng(1)
    cu = np.array([0, 30, 30, 75, 100])
    w = rng.integers(0, 1000, 100)
    a = sch.select_schedule(cu, w, seed=4, step=2, rollout_id_base=10)
    b = sch.select_schedule(cu[2:] - 30, w[30:], seed=4, step=2, rollout_id_base=12)
    assert np.array_equal(a["cut_len"][2:], b["cut_len"]) and np.array_equal(a["mask"][30:], b["mask"])
    c = sch.select_schedule(cu, w, seed=4, step=3, rollout_id_base=10)
    assert not np.array_equal(a["cut_len"], c["cut_len"])
    # mask is the prefix indicator of Eq. 7
    for i in range(4):
        seg = a["mask"][cu[i]:cu[i + 1]]
        assert seg.sum() == a["cut_len"][i] and seg[:a["cut_len"][i]].all()


# ---------------------------------------------------------------- Prop. 1 and App. B.1 with a general q

def test_prop1_general_schedule_exhaustive_enumeration():
    b = tiny_batch(41, [5, 4, 3])
    w = np.array([1, 0, 3, 2, 5,   2, 2, 0, 1,   0, 0, 4])
    ft = drivers.full_token(b)
    e = drivers.enumerate_schedule(b, w)
    assert abs(e["prob"] - 1) < 1e-12
    assert abs(e["loss"] - ft["loss"]) < 1e-12
    assert np.abs(e["dH"] - ft["dH"]).max() < 1e-12
    assert np.abs(e["dW"] - ft["dW"]).max() < 1e-12


def test_uniform_weights_reproduce_the_uniform_rpc_enumeration():
    b = tiny_batch(42, [4, 3])
    e1 = drivers.enumerate_schedule(b, np.ones(7, dtype=np.int64))
    e2 = drivers.enumerate_rpc(b, C=1)
    assert np.isclose(e1["loss_sq"], e2["loss_sq"], rtol=1e-13) and np.isclose(e1["loss"], e2["loss"], rtol=1e-13)


def test_stopping_time_variance_with_general_q():
    T = 8
    b = tiny_batch(43, [T])
    a = [2, 0, 1, 4, 0, 3, 1, 2]
    e = drivers.enumerate_schedule(b, np.array(a))
    var_enum = e["loss_sq"] - e["loss"] ** 2
    assert np.isclose(var_enum, drivers.var_rpc_stopping(_token_losses(b), sch.schedule_pi(a), sch.schedule_q(a)),
                      rtol=1e-10)


def test_mask_covariance_is_p_t_times_one_minus_p_s():
    a = [1, 3, 0, 2, 4]
    q, pi = sch.schedule_q(a), sch.schedule_pi(a)
    T = len(a)
    for s in range(T):
        for t in range(s, T):
            # E[m_s m_t] = Pr(L >= t) for s <= t
            cov = sum(q[l] for l in range(T) if l >= t) - pi[s] * pi[t]
            assert np.isclose(cov, pi[t] * (1 - pi[s]), atol=1e-15)


# ---------------------------------------------------------------- Poisson sampling (Sec. 3.1)

def test_constant_probability_reproduces_urs_draw_for_draw():
    for p in (0.25, 0.5, 0.8, 1.0):
        m1 = sch.poisson_mask(np.full(1000, p), seed=8, step=3, rollout_id=17)
        assert np.array_equal(m1, sel.urs_mask(1000, p, seed=8, step=3, rollout_id=17))


def test_probability_zero_never_keeps_and_one_always_keeps():
    pi = np.tile([0.0, 1.0], 500)
    m = sch.poisson_mask(pi, seed=1, step=0, rollout_id=0)
    assert not m[0::2].any() and m[1::2].all()
    with pytest.raises(ValueError):
        sch.poisson_threshold(1.0000001)


def test_keep_rate_per_probability_level():
    levels = np.array([0.1, 0.35, 0.9])
    pi = np.tile(levels, 200000)
    m = sch.poisson_mask(pi, seed=77, step=0, rollout_id=3)
    for j, p in enumerate(levels):
        k, n = int(m[j::3].sum()), 200000
        assert abs(k - n * p) < 5 * math.sqrt(n * p * (1 - p))


def test_prop1_heterogeneous_probabilities_exhaustive_enumeration():
    b = tiny_batch(44, [5, 4])
    pi = np.array([0.9, 0.2, 0.5, 1.0, 0.35, 0.6, 0.75, 0.15, 0.5])
    ft = drivers.full_token(b)
    e = drivers.enumerate_poisson(b, pi)
    assert abs(e["prob"] - 1) < 1e-12
    assert abs(e["loss"] - ft["loss"]) < 1e-12
    assert np.abs(e["dW"] - ft["dW"]).max() < 1e-12 and np.abs(e["dH"] - ft["dH"]).max() < 1e-12


def test_independent_mask_variance_with_heterogeneous_probabilities():
    b = tiny_batch(45, [8])
    pi = np.array([0.9, 0.2, 0.5, 1.0, 0.35, 0.6, 0.75, 0.15])
    e = drivers.enumerate_poisson(b, pi)
    assert np.isclose(e["loss_sq"] - e["loss"] ** 2, drivers.var_independent(_token_losses(b), pi), rtol=1e-10)


# ---------------------------------------------------------------- weights, compaction

def test_weight_from_probability_agrees_with_the_scheme_closed_forms():
    # same factor as select.ht_weight (one rounding apart at most: two fp64 operations instead of one)
    for T, t, C in ((9, 5, 1), (3000, 2999, 100), (17, 3, 4)):
        pi = sel.inclusion_prob(sel.RPC, T, C=C)[t - 1]
        w1, w2 = sch.ht_weight_pi(T, pi, 128), sel.ht_weight(sel.RPC, T, t, 128, C=C)
        assert abs(float(w1) - float(w2)) <= np.spacing(np.float32(w2))
    assert sch.ht_weight_pi(10, 0.5, 4) == np.float32(1 / 20)


def test_compact_pi_matches_scheme_compaction_on_the_index_outputs():
    cu = np.array([0, 0, 37, 37, 100, 101])
    d = sel.select(cu, sel.URS, p=0.5, seed=3, step=1)
    c1 = sel.compact(d["mask"], cu, 5, sel.URS, p=0.5)
    c2 = sch.compact_pi(d["mask"], d["pi"], cu, 5)
    for k in ("kept_idx", "kept_seq", "cu_kept", "kept_w"):      # p = .5: weights agree exactly as well
        assert np.array_equal(c1[k], c2[k]), k
    # sum_t m_t /(T p_t) has expectation 1: enumeration for one short rollout
    pi = np.array([1.0, 0.5, 0.25])
    tot = 0.0
    for bits in range(8):
        m = np.array([(bits >> j) & 1 for j in range(3)], dtype=bool)
        prob = float(np.prod(np.where(m, pi, 1 - pi)))
        tot += prob * float(sch.compact_pi(m, pi, [0, 3], 1)["kept_w"].astype(np.float64).sum())
    assert abs(tot - 1.0) < 1e-6


# ---------------------------------------------------------------- prefix packing

def _reference_rows(P, T, L):
    # independent construction: label every full-input row (rollout, j) and slice per rollout
    rows, off = [], 0
    full = []
    for i in range(len(T)):
        full.append([(i, j) for j in range(P[i] + T[i])])
    return [lab for i in range(len(T)) for lab in full[i][:P[i] + L[i]]], full


@pytest.mark.parametrize("shift", [0, 1])
def test_prefix_pack_against_per_rollout_slicing(shift):
    rng = np.random.default_rng(9)
    T = np.array([5, 0, 9, 1, 30])
    P = np.array([3, 2, 1, 4, 7])
    L = np.array([2, 0, 9, 0, 11])
    cu = np.concatenate([[0], np.cumsum(T)])
    out = sch.prefix_pack(P, cu, L, shift)
    labels, full = _reference_rows(P, T, L)
    flat = [lab for seq in full for lab in seq]
    assert [flat[s] for s in out["src_idx"]] == labels
    assert [lab[1] for lab in labels] == out["position_ids"].tolist()
    assert out["cu_packed"].tolist() == np.concatenate([[0], np.cumsum(P + L)]).tolist()
    assert out["total"] == int((P + L).sum()) and out["max_len"] == int((P + L).max())
    # the scoring row of kept response token (i, t0) is `shift` rows before that token's own row
    k = 0
    for i in range(len(T)):
        for t0 in range(L[i]):
            assert labels[out["loss_row"][k] + shift] == (i, P[i] + t0)
            assert out["cu_packed"][i] <= out["loss_row"][k] < out["cu_packed"][i + 1]
            k += 1
    assert k == len(out["loss_row"]) == L.sum()


def test_prefix_pack_without_prompts_and_full_cut_is_the_identity():
    T = np.array([4, 6, 1])
    cu = np.concatenate([[0], np.cumsum(T)])
    out = sch.prefix_pack(None, cu, T, 0)
    assert out["src_idx"].tolist() == list(range(11)) == out["loss_row"].tolist()
    assert out["position_ids"].tolist() == [0, 1, 2, 3, 0, 1, 2, 3, 4, 5, 0]
    with pytest.raises(ValueError):
        sch.prefix_pack(None, cu, T, 1)                          # no state precedes the first response token
    with pytest.raises(ValueError):
        sch.prefix_pack(None, cu, T + 1, 0)


def test_prefix_pack_rows_scale_with_the_cut_as_the_paper_states():
    # uniform cuts keep about half of the response rows (Sec. 4: E[L] ~ T/2)
    T = np.full(400, 1000)
    cu = np.concatenate([[0], np.cumsum(T)])
    d = sel.select(cu, sel.RPC, C=1, seed=6, step=0)
    out = sch.prefix_pack(np.full(400, 10), cu, d["cut_len"], 1)
    resp_rows = out["total"] - 400 * 10
    assert abs(resp_rows / T.sum() - 0.5) < 0.05
    assert len(out["loss_row"]) == int(d["mask"].sum())


# ------------------------------------------------- zero-advantage rollouts ----

def test_schedule_and_poisson_dropping_zero_advantage_rollouts_leaves_the_estimate_unchanged():
    # Eq. 3 with A = 0: S = 0 and dS/dlogp = 0 at every token of the rollout, whatever the ratio
    b = tiny_batch(61, [5, 4, 6, 3])
    b["adv"] = np.array([0.7, 0.0, -1.2, 0.0])
    cu = b["cu_seqlens"]
    N = int(cu[-1])
    rng = np.random.default_rng(3)
    w = rng.integers(1, 50, N).astype(np.uint32)
    keep_all = sch.select_schedule(cu, w, seed=4, step=2)
    dropped = sch.select_schedule(cu, w, seed=4, step=2, drop_zero_adv=b["adv"])
    assert dropped["cut_len"].tolist() == [keep_all["cut_len"][0], 0, keep_all["cut_len"][2], 0]
    assert not dropped["mask"][cu[1]:cu[2]].any() and not dropped["mask"][cu[3]:cu[4]].any()
    for i in (0, 2):                                           # the other rollouts draw exactly as before
        assert np.array_equal(dropped["mask"][cu[i]:cu[i + 1]], keep_all["mask"][cu[i]:cu[i + 1]])
    assert np.array_equal(dropped["pi"], keep_all["pi"])       # survival functions (and weights) unchanged
    e1 = drivers.estimate(b, keep_all["mask"], keep_all["pi"])
    e2 = drivers.estimate(b, dropped["mask"], dropped["pi"])
    assert abs(e1["loss"] - e2["loss"]) < 1e-15
    assert np.abs(e1["dW"] - e2["dW"]).max() < 1e-15 and np.abs(e1["dH"] - e2["dH"]).max() < 1e-15

    pi = 0.2 + 0.8 * rng.random(N)
    m_all = sch.select_poisson(cu, pi, seed=9, step=1)
    m_drop = sch.select_poisson(cu, pi, seed=9, step=1, drop_zero_adv=b["adv"])
    assert m_all[cu[1]:cu[2]].any() and not m_drop[cu[1]:cu[2]].any() and not m_drop[cu[3]:cu[4]].any()
    for i in (0, 2):
        assert np.array_equal(m_drop[cu[i]:cu[i + 1]], m_all[cu[i]:cu[i + 1]])
    e1 = drivers.estimate(b, m_all, pi)
    e2 = drivers.estimate(b, m_drop, pi)
    assert abs(e1["loss"] - e2["loss"]) < 1e-15 and np.abs(e1["dW"] - e2["dW"]).max() < 1e-15
    # negative control: with a KL term the dropped tokens would have contributed
    bk = dict(b, ref_logp=b["old_logp"] + 0.3, beta_kl=0.5, kl_kind=grpo.KL_NONNEG)
    assert abs(drivers.estimate(bk, m_all, pi)["loss"] - drivers.estimate(bk, m_drop, pi)["loss"]) > 1e-4
    # no advantages given, or none of them zero: nothing changes
    same = sch.select_schedule(cu, w, seed=4, step=2, drop_zero_adv=np.array([0.7, 0.1, -1.2, 3.0]))
    assert np.array_equal(same["mask"], keep_all["mask"]) and np.array_equal(same["cut_len"], keep_all["cut_len"])
