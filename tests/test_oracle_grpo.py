"""Pins for oracle.grpo and oracle.drivers: Eq. 1-5 hand cases, library
routines on the textbook special case, finite differences, Prop. 1 by exhaustive
enumeration, closed-form variances (Sec. 3.1, App. B.1, B.4), Monte Carlo."""
import math

import numpy as np
import pytest
import torch
from scipy.special import log_softmax as scipy_log_softmax

from oracle import drivers, grpo
from oracle import select as sel


def tiny_batch(seed, lengths, H=8, V=16, noise=0.15):
    rng = np.random.default_rng(seed)
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    N = int(cu[-1])
    b = dict(cu_seqlens=cu, hidden=rng.standard_normal((N, H)), W=rng.standard_normal((V, H)) * 0.3,
             ids=rng.integers(0, V, N), adv=rng.standard_normal(len(lengths)))
    b["old_logp"] = grpo.token_logp(b["hidden"], b["W"], b["ids"]) + rng.standard_normal(N) * noise
    return b


# ------------------------------------------------------------ Eq. 2 ----

def test_advantage_hand_values():
    A = grpo.advantages([[1, 0, 0, 1]], eps_adv=1e-6)
    assert np.allclose(A, np.array([[0.5, -0.5, -0.5, 0.5]]) / (0.5 + 1e-6), rtol=1e-15)
    A = grpo.advantages([[1, 0, 0, 0]], eps_adv=1e-6)
    s = math.sqrt(3) / 4           # population std of {1,0,0,0}
    assert np.allclose(A, [[0.75 / (s + 1e-6), *[-0.25 / (s + 1e-6)] * 3]], rtol=1e-14)
    # all-equal rewards: zero advantage for the whole group
    assert (grpo.advantages([[1, 1, 1, 1], [0, 0, 0, 0]]) == 0).all()
    # groups are normalised independently
    A2 = grpo.advantages([[1, 0], [5, 3]], eps_adv=0.0)
    assert np.allclose(A2, [[1, -1], [1, -1]])


# ------------------------------------------------------------ Eq. 3 ----

def test_clipped_surrogate_hand_cases():
    eps = 0.2
    lr = lambda r: math.log(r)
    # A>0, r above the trust region: S = (1+eps) A, no gradient
    r, S, g = grpo.surrogate([lr(1.5)], [0.0], [2.0], eps, eps)
    assert np.isclose(S[0], 1.2 * 2.0) and g[0] == 0.0
    # A<0, r below the trust region: S = (1-eps) A, no gradient
    r, S, g = grpo.surrogate([lr(0.5)], [0.0], [-2.0], eps, eps)
    assert np.isclose(S[0], 0.8 * -2.0) and g[0] == 0.0
    # A>0, r below: unclipped branch is the min
    r, S, g = grpo.surrogate([lr(0.5)], [0.0], [2.0], eps, eps)
    assert np.isclose(S[0], 1.0) and np.isclose(g[0], 1.0)
    # A<0, r above: unclipped (more negative) branch is the min
    r, S, g = grpo.surrogate([lr(1.5)], [0.0], [-2.0], eps, eps)
    assert np.isclose(S[0], -3.0) and np.isclose(g[0], -3.0)
    # inside the region
    r, S, g = grpo.surrogate([lr(1.1)], [0.0], [-1.0], eps, eps)
    assert np.isclose(S[0], -1.1) and np.isclose(g[0], -1.1)
    # zero advantage
    r, S, g = grpo.surrogate([lr(1.1)], [0.0], [0.0], eps, eps)
    assert S[0] == 0.0 and g[0] == 0.0
    # asymmetric clip range
    r, S, g = grpo.surrogate([lr(1.25)], [0.0], [1.0], 0.2, 0.3)
    assert np.isclose(S[0], 1.25) and np.isclose(g[0], 1.25)


def test_surrogate_gradient_is_derivative_of_S():
    rng = np.random.default_rng(3)
    logp = rng.standard_normal(400) * 0.3
    old = np.zeros(400)
    A = rng.standard_normal(400)
    _, S, g = grpo.surrogate(logp, old, A, 0.2, 0.2)
    d = 1e-7
    _, Sp, _ = grpo.surrogate(logp + d, old, A, 0.2, 0.2)
    _, Sm, _ = grpo.surrogate(logp - d, old, A, 0.2, 0.2)
    fd = (Sp - Sm) / (2 * d)
    r = np.exp(logp)
    away = (np.abs(r - 1.2) > 1e-4) & (np.abs(r - 0.8) > 1e-4)
    assert away.sum() > 380
    assert np.allclose(fd[away], g[away], rtol=1e-6, atol=1e-8)
    assert (g == 0).sum() > 20          # the clipped branch is exercised


# ---------------------------------------------- soft-max head, library ----

def test_log_softmax_against_scipy():
    rng = np.random.default_rng(0)
    Z = rng.standard_normal((7, 33)) * 10
    assert np.allclose(grpo.log_softmax_rows(Z), scipy_log_softmax(Z, axis=1), rtol=1e-13, atol=1e-13)
    Zbig = Z + 1e4                       # shift invariance / no overflow
    assert np.allclose(grpo.log_softmax_rows(Zbig), scipy_log_softmax(Z, axis=1), rtol=1e-9, atol=1e-9)


def test_on_policy_unclipped_case_is_weighted_cross_entropy():
    # with old_logp = logp (r = 1) and no clipping, d loss / d theta equals the
    # gradient of sum_k w_k A_k * CE_k: check against torch's cross_entropy + autograd
    b = tiny_batch(1, [6, 5], H=8, V=16)
    N = 11
    seq = np.repeat([0, 1], [6, 5])
    w = np.random.default_rng(2).random(N) + 0.1
    old = grpo.token_logp(b["hidden"], b["W"], b["ids"])
    out = grpo.loss_and_grads(b["hidden"], b["W"], b["ids"], old, b["adv"][seq], w, 1e9, 1e9)
    Ht = torch.tensor(b["hidden"], dtype=torch.float64, requires_grad=True)
    Wt = torch.tensor(b["W"], dtype=torch.float64, requires_grad=True)
    ce = torch.nn.functional.cross_entropy(Ht @ Wt.T, torch.tensor(b["ids"]), reduction="none")
    (torch.tensor(w * b["adv"][seq]) * ce).sum().backward()
    assert np.allclose(out["dH"], Ht.grad.numpy(), rtol=1e-11, atol=1e-13)
    assert np.allclose(out["dW"], Wt.grad.numpy(), rtol=1e-11, atol=1e-13)
    assert np.isclose(out["loss"], -(w * b["adv"][seq]).sum())      # r = 1  =>  S = A
    assert np.allclose(out["logp"], -ce.detach().numpy(), rtol=1e-12)


def test_gradients_against_autograd_with_clipping_active():
    # full objective re-expressed with torch ops (min / clamp), differentiated by autograd
    b = tiny_batch(4, [7, 4, 5], H=8, V=16, noise=0.25)
    N = 16
    seq = np.repeat([0, 1, 2], [7, 4, 5])
    w = 1.0 / (3 * np.array([7, 4, 5])[seq])
    out = grpo.loss_and_grads(b["hidden"], b["W"], b["ids"], b["old_logp"], b["adv"][seq], w, 0.2, 0.2)
    Ht = torch.tensor(b["hidden"], requires_grad=True)
    Wt = torch.tensor(b["W"], requires_grad=True)
    lp = torch.log_softmax(Ht @ Wt.T, dim=1)[torch.arange(N), torch.tensor(b["ids"])]
    r = torch.exp(lp - torch.tensor(b["old_logp"]))
    A = torch.tensor(b["adv"][seq])
    S = torch.minimum(r * A, torch.clamp(r, 0.8, 1.2) * A)
    loss = -(torch.tensor(w) * S).sum()
    loss.backward()
    assert np.isclose(out["loss"], loss.item(), rtol=1e-13)
    assert np.allclose(out["dH"], Ht.grad.numpy(), rtol=1e-10, atol=1e-14)
    assert np.allclose(out["dW"], Wt.grad.numpy(), rtol=1e-10, atol=1e-14)
    clipped = ((out["r"] > 1.2) & (A.numpy() > 0)) | ((out["r"] < 0.8) & (A.numpy() < 0))
    assert clipped.sum() >= 2 and (~clipped).sum() >= 2


def test_gradients_against_central_finite_differences():
    b = tiny_batch(7, [5, 6], H=6, V=12, noise=0.1)
    seq = np.repeat([0, 1], [5, 6])
    w = 1.0 / (2 * np.array([5, 6])[seq])
    args = (b["ids"], b["old_logp"], b["adv"][seq], w, 0.2, 0.2)
    out = grpo.loss_and_grads(b["hidden"], b["W"], *args)
    d = 1e-6
    rng = np.random.default_rng(0)
    for _ in range(25):
        k, h = rng.integers(0, 11), rng.integers(0, 6)
        Hp, Hm = b["hidden"].copy(), b["hidden"].copy()
        Hp[k, h] += d
        Hm[k, h] -= d
        fd = (grpo.objective_value(Hp, b["W"], *args) - grpo.objective_value(Hm, b["W"], *args)) / (2 * d)
        assert abs(fd - out["dH"][k, h]) < 1e-8
        v = rng.integers(0, 12)
        Wp, Wm = b["W"].copy(), b["W"].copy()
        Wp[v, h] += d
        Wm[v, h] -= d
        fd = (grpo.objective_value(b["hidden"], Wp, *args) - grpo.objective_value(b["hidden"], Wm, *args)) / (2 * d)
        assert abs(fd - out["dW"][v, h]) < 1e-8


def test_empty_token_set():
    out = grpo.loss_and_grads(np.zeros((0, 4)), np.ones((5, 4)), [], [], [], [])
    assert out["loss"] == 0.0 and out["dW"].shape == (5, 4) and not out["dW"].any()


# ------------------------------------------------ Eq. 5 / Eq. 6 / Prop. 1 ----

def test_full_token_objective_is_sequence_then_group_mean():
    # Eq. 5 written out rollout by rollout
    b = tiny_batch(11, [3, 6, 4])
    ft = drivers.full_token(b)
    logp = grpo.token_logp(b["hidden"], b["W"], b["ids"])
    J = 0.0
    for i in range(3):
        sl = slice(b["cu_seqlens"][i], b["cu_seqlens"][i + 1])
        _, S, _ = grpo.surrogate(logp[sl], b["old_logp"][sl], np.full(sl.stop - sl.start, b["adv"][i]), 0.2, 0.2)
        J += S.mean() / 3
    assert np.isclose(ft["loss"], -J, rtol=1e-13)


def test_p_equal_one_and_no_cut_reproduce_full_token_exactly():
    b = tiny_batch(12, [9, 14, 1])
    ft = drivers.full_token(b)
    for scheme, kw in [(sel.URS, dict(p=1.0)), (sel.RPC, dict(C=10 ** 6)), (sel.FULL, {}), (sel.DET, dict(beta=1.0))]:
        d = sel.select(b["cu_seqlens"], scheme, seed=5, **kw)
        assert d["mask"].all()
        est = drivers.estimate(b, d["mask"], d["pi"])
        assert est["loss"] == ft["loss"]
        assert np.array_equal(est["dH"], ft["dH"]) and np.array_equal(est["dW"], ft["dW"])


def test_prop1_urs_exhaustive_enumeration():
    b = tiny_batch(21, [4, 5])                      # 2^9 masks
    ft = drivers.full_token(b)
    for p in (0.5, 0.3):
        e = drivers.enumerate_urs(b, p)
        assert abs(e["prob"] - 1) < 1e-12
        assert abs(e["loss"] - ft["loss"]) < 1e-12
        assert np.abs(e["dH"] - ft["dH"]).max() < 1e-12
        assert np.abs(e["dW"] - ft["dW"]).max() < 1e-12


@pytest.mark.parametrize("C", [1, 3])
def test_prop1_rpc_exhaustive_enumeration(C):
    b = tiny_batch(22, [6, 5, 2])
    ft = drivers.full_token(b)
    e = drivers.enumerate_rpc(b, C=C)
    assert abs(e["prob"] - 1) < 1e-12
    assert abs(e["loss"] - ft["loss"]) < 1e-12
    assert np.abs(e["dH"] - ft["dH"]).max() < 1e-12
    assert np.abs(e["dW"] - ft["dW"]).max() < 1e-12


def test_det_trunc_is_biased_negative_control():
    b = tiny_batch(23, [6, 5])
    ft = drivers.full_token(b)
    dt = drivers.det_trunc(b, 0.5)
    assert np.abs(dt["dW"] - ft["dW"]).max() > 1e-3 * np.abs(ft["dW"]).max()
    assert (dt["dH"][3:6] == 0).all() and (dt["dH"][6 + 2:] == 0).all()
    # and a wrong weight (forgetting 1/p) must fail the enumeration test
    e = drivers.enumerate_urs(tiny_batch(21, [3, 3]), 0.5)
    assert abs(0.5 * e["loss"] - drivers.full_token(tiny_batch(21, [3, 3]))["loss"]) > 1e-6


# ----------------------------------------------------------- variances ----

def _token_losses(b):
    logp = grpo.token_logp(b["hidden"], b["W"], b["ids"])
    seq = np.repeat(np.arange(len(b["adv"])), np.diff(b["cu_seqlens"]))
    return grpo.surrogate(logp, b["old_logp"], b["adv"][seq], 0.2, 0.2)[1]


def test_independent_mask_variance_closed_form():
    b = tiny_batch(31, [8])
    Lt = _token_losses(b)
    p = 0.4
    e = drivers.enumerate_urs(b, p)
    var_enum = e["loss_sq"] - e["loss"] ** 2
    assert np.isclose(var_enum, drivers.var_independent(Lt, np.full(8, p)), rtol=1e-10)


@pytest.mark.parametrize("C", [1, 4])
def test_rpc_stopping_time_variance_closed_form(C):
    T = 9
    b = tiny_batch(32, [T])
    Lt = _token_losses(b)
    pi = sel.inclusion_prob(sel.RPC, T, C=C)
    Ci = sel.rpc_min_cut(T, C)
    q = np.array([1.0 / (T - Ci + 1) if l >= Ci else 0.0 for l in range(1, T + 1)])
    e = drivers.enumerate_rpc(b, C=C)
    var_enum = e["loss_sq"] - e["loss"] ** 2
    assert np.isclose(var_enum, drivers.var_rpc_stopping(Lt, pi, q), rtol=1e-10)
    # positive mask correlation: RPC variance exceeds the independent-mask value
    # only through the covariance terms; with one token both vanish
    assert drivers.var_rpc_stopping(Lt[:1], [1.0], [1.0]) == 0.0


def test_urs_second_moment_inflation():
    # E|| (m/p) g ||^2 = ||g||^2 / p for one token (Sec. 3.1)
    b = tiny_batch(33, [1])
    g = drivers.full_token(b)["dW"]
    for p in (0.5, 0.25):
        pi = np.array([p])
        second = p * (drivers.estimate(b, [True], pi)["dW"] ** 2).sum() + (1 - p) * 0.0
        assert np.isclose(second, (g ** 2).sum() / p, rtol=1e-12)


def test_ht_value_unbiased_by_enumeration():
    rng = np.random.default_rng(0)
    Lt = rng.standard_normal(6)
    pi = np.array([1.0, 0.9, 0.7, 0.5, 0.3, 0.2])
    tot = 0.0
    for bits in range(64):
        m = np.array([(bits >> k) & 1 for k in range(6)], dtype=bool)
        tot += np.prod(np.where(m, pi, 1 - pi)) * drivers.ht_value(Lt, m, pi)
    assert abs(tot - Lt.mean()) < 1e-13


# ---------------------------------------------------------- Monte Carlo ----

@pytest.mark.parametrize("scheme,kw", [(sel.URS, dict(p=0.5)), (sel.RPC, dict(C=1))])
def test_monte_carlo_mean_converges_to_full_token(scheme, kw):
    b = tiny_batch(41, [7, 9], H=4, V=8)
    ft = drivers.full_token(b)
    K = 3000
    seeds = range(1000, 1000 + K)
    sums = None
    sq = None
    for s in seeds:
        d = sel.select(b["cu_seqlens"], scheme, seed=s, **kw)
        est = drivers.estimate(b, d["mask"], d["pi"])
        v = np.concatenate([[est["loss"]], est["dW"].ravel()])
        sums = v if sums is None else sums + v
        sq = v * v if sq is None else sq + v * v
    mean = sums / K
    std = np.sqrt(np.maximum(sq / K - mean ** 2, 0))
    ref = np.concatenate([[ft["loss"]], ft["dW"].ravel()])
    assert (np.abs(mean - ref) <= 5 * std / math.sqrt(K) + 1e-12).all()
    # the driver form over the same seeds reproduces the running sums kept above
    mc = drivers.monte_carlo(b, scheme, list(seeds), **kw)
    assert np.isclose(mc["prob"], 1.0, rtol=0, atol=1e-12)
    assert np.allclose(np.concatenate([[mc["loss"]], mc["dW"].ravel()]), mean, rtol=1e-11, atol=1e-15)
    assert np.isclose(mc["loss_sq"], sq[0] / K, rtol=1e-11)
    assert (np.abs(np.concatenate([[mc["loss"]], mc["dW"].ravel()]) - ref) <= 5 * std / math.sqrt(K) + 1e-12).all()


def test_monte_carlo_driver_on_a_hand_enumerable_case():
    # one rollout of two tokens under URS p = 1/2: the driver's mean over seeds is the average of the
    # per-seed estimates, each of which is one of the four masks' estimates; and with p = 1 every
    # draw is the full-token value
    b = tiny_batch(43, [2], H=4, V=8)
    pi = np.full(2, 0.5)
    by_mask = {bits: drivers.estimate(b, np.array(bits), pi) for bits in
               [(False, False), (False, True), (True, False), (True, True)]}
    seeds = list(range(40))
    want_loss, want_dW, want_sq = 0.0, 0.0, 0.0
    seen = set()
    for s in seeds:
        m = tuple(bool(x) for x in sel.select(b["cu_seqlens"], sel.URS, p=0.5, seed=s)["mask"])
        seen.add(m)
        want_loss += by_mask[m]["loss"] / len(seeds)
        want_dW = want_dW + by_mask[m]["dW"] / len(seeds)
        want_sq += by_mask[m]["loss"] ** 2 / len(seeds)
    assert len(seen) == 4                                   # every mask occurs among the draws
    mc = drivers.monte_carlo(b, sel.URS, seeds, p=0.5)
    assert np.isclose(mc["loss"], want_loss, rtol=1e-12) and np.isclose(mc["loss_sq"], want_sq, rtol=1e-12)
    assert np.allclose(mc["dW"], want_dW, rtol=1e-12, atol=1e-18)
    ft = drivers.full_token(b)
    one = drivers.monte_carlo(b, sel.URS, [1, 2, 3], p=1.0)
    assert np.isclose(one["loss"], ft["loss"], rtol=1e-13) and np.allclose(one["dW"], ft["dW"], rtol=1e-12, atol=1e-18)
