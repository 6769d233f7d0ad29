"""Pins for the KL term of Eq. 4 (sampled-token forms named in its footnote) and
the per-token entropy (the quantity of the entropy figure in Sec. 5) in
oracle.grpo."""
import numpy as np
import pytest
import torch
from scipy.special import softmax
from scipy.stats import entropy as scipy_entropy

from oracle import drivers, grpo
from test_oracle_grpo import tiny_batch


def _with_ref(b, seed, beta, kind, spread=0.3):
    rng = np.random.default_rng(seed)
    b = dict(b)
    logp = grpo.token_logp(b["hidden"], b["W"], b["ids"])
    b["ref_logp"] = logp + rng.standard_normal(len(logp)) * spread
    b["beta_kl"], b["kl_kind"] = beta, kind
    return b


# ---------------------------------------------------------------- entropy

def test_entropy_against_scipy_and_closed_forms():
    rng = np.random.default_rng(0)
    Z = rng.standard_normal((7, 33)) * 2.0
    H = grpo.entropy_rows(grpo.log_softmax_rows(Z))
    for k in range(7):
        assert np.isclose(H[k], scipy_entropy(softmax(Z[k])), rtol=1e-12)
    # uniform policy: ln V;  a policy concentrated on one token: ~0
    assert np.allclose(grpo.entropy_rows(grpo.log_softmax_rows(np.zeros((2, 50)))), np.log(50), rtol=1e-14)
    peaked = np.zeros((1, 50)); peaked[0, 3] = 60.0
    assert grpo.entropy_rows(grpo.log_softmax_rows(peaked))[0] < 1e-20 * 1e3
    # two-point distribution (p, 1-p): -p ln p - (1-p) ln(1-p)
    p = 0.2
    two = np.log(np.array([[p, 1 - p]]))
    assert np.isclose(grpo.entropy_rows(grpo.log_softmax_rows(two))[0], -p * np.log(p) - (1 - p) * np.log(1 - p))


def test_loss_and_grads_reports_entropy_of_each_token():
    b = tiny_batch(3, [4, 3])
    out = grpo.loss_and_grads(b["hidden"], b["W"], b["ids"], b["old_logp"], np.ones(7), np.ones(7))
    P = softmax(b["hidden"] @ b["W"].T, axis=1)
    assert np.allclose(out["entropy"], [scipy_entropy(P[k]) for k in range(7)], rtol=1e-12)


# ---------------------------------------------------------------- KL forms

def test_kl_forms_zero_at_equal_policies_and_sign():
    lp = np.array([-1.0, -3.0])
    for kind in (grpo.KL_LOG_RATIO, grpo.KL_NONNEG):
        kl, dkl = grpo.kl_term(lp, lp, kind)
        assert np.array_equal(kl, np.zeros(2))
    assert np.array_equal(grpo.kl_term(lp, lp, grpo.KL_LOG_RATIO)[1], np.ones(2))
    assert np.array_equal(grpo.kl_term(lp, lp, grpo.KL_NONNEG)[1], np.zeros(2))   # minimum of a non-negative term
    ref = lp + np.array([0.7, -0.4])
    assert (grpo.kl_term(lp, ref, grpo.KL_NONNEG)[0] > 0).all()
    assert np.allclose(grpo.kl_term(lp, ref, grpo.KL_LOG_RATIO)[0], [-0.7, 0.4])
    with pytest.raises(ValueError):
        grpo.kl_term(lp, ref, 7)


@pytest.mark.parametrize("kind", [grpo.KL_LOG_RATIO, grpo.KL_NONNEG])
def test_sampled_token_forms_are_unbiased_for_the_true_kl(kind):
    # E_{o ~ pi_theta}[KL_k(o)] = D_KL(pi_theta || pi_ref): exact sum over the vocabulary
    rng = np.random.default_rng(1)
    p = softmax(rng.standard_normal(40))
    q = softmax(rng.standard_normal(40))
    kl_tok, _ = grpo.kl_term(np.log(p), np.log(q), kind)
    assert np.isclose(np.sum(p * kl_tok), scipy_entropy(p, q), rtol=1e-12)       # scipy: sum p log(p/q)
    assert not np.isclose(np.sum(p * kl_tok), scipy_entropy(q, p), rtol=1e-3)    # not the reverse direction


@pytest.mark.parametrize("kind", [grpo.KL_LOG_RATIO, grpo.KL_NONNEG])
def test_derivative_of_kl_term_by_finite_differences(kind):
    lp, ref, d = np.array([-2.0, -0.5, -7.0]), np.array([-1.5, -0.9, -7.2]), 1e-6
    _, dkl = grpo.kl_term(lp, ref, kind)
    fd = (grpo.kl_term(lp + d, ref, kind)[0] - grpo.kl_term(lp - d, ref, kind)[0]) / (2 * d)
    assert np.allclose(dkl, fd, atol=1e-8)


# ---------------------------------------------------------------- Eq. 4 in the loss

def test_beta_zero_changes_nothing():
    b = tiny_batch(5, [4, 5])
    args = (b["hidden"], b["W"], b["ids"], b["old_logp"], np.repeat(b["adv"], [4, 5]), np.full(9, 0.1))
    a = grpo.loss_and_grads(*args)
    c = grpo.loss_and_grads(*args, ref_logp=b["old_logp"] - 1.0, beta_kl=0.0, kl_kind=grpo.KL_NONNEG)
    assert a["loss"] == c["loss"] and np.array_equal(a["dW"], c["dW"]) and np.array_equal(a["dH"], c["dH"])


@pytest.mark.parametrize("kind", [grpo.KL_LOG_RATIO, grpo.KL_NONNEG])
def test_loss_is_surrogate_minus_beta_kl(kind):
    b = _with_ref(tiny_batch(6, [4, 5]), 1, 0.3, kind)
    adv_tok, w = np.repeat(b["adv"], [4, 5]), np.full(9, 0.1)
    out = grpo.loss_and_grads(b["hidden"], b["W"], b["ids"], b["old_logp"], adv_tok, w, ref_logp=b["ref_logp"],
                              beta_kl=0.3, kl_kind=kind)
    base = grpo.loss_and_grads(b["hidden"], b["W"], b["ids"], b["old_logp"], adv_tok, w)
    kl = grpo.kl_term(base["logp"], b["ref_logp"], kind)[0]
    assert np.isclose(out["loss"], base["loss"] + 0.3 * np.sum(w * kl), rtol=1e-13)
    assert np.allclose(out["kl"], kl)


@pytest.mark.parametrize("kind", [grpo.KL_LOG_RATIO, grpo.KL_NONNEG])
def test_gradients_with_kl_against_autograd_and_finite_differences(kind):
    b = _with_ref(tiny_batch(8, [5, 6], H=6, V=12, noise=0.3), 2, 0.25, kind)
    seq = np.repeat([0, 1], [5, 6])
    w = 1.0 / (2 * np.array([5, 6])[seq])
    kw = dict(ref_logp=b["ref_logp"], beta_kl=0.25, kl_kind=kind)
    args = (b["ids"], b["old_logp"], b["adv"][seq], w, 0.2, 0.2)
    out = grpo.loss_and_grads(b["hidden"], b["W"], *args, **kw)
    # autograd on the same formula written with torch ops
    Ht = torch.tensor(b["hidden"], requires_grad=True)
    Wt = torch.tensor(b["W"], requires_grad=True)
    logp = torch.log_softmax(Ht @ Wt.T, dim=1)[torch.arange(11), torch.tensor(b["ids"])]
    A = torch.tensor(b["adv"][seq])
    r = torch.exp(logp - torch.tensor(b["old_logp"]))
    S = torch.minimum(r * A, torch.clamp(r, 0.8, 1.2) * A)
    d = torch.tensor(b["ref_logp"]) - logp
    kl = -d if kind == grpo.KL_LOG_RATIO else torch.exp(d) - d - 1
    loss = -(torch.tensor(w) * (S - 0.25 * kl)).sum()
    loss.backward()
    assert np.isclose(out["loss"], loss.item(), rtol=1e-13)
    assert np.allclose(out["dH"], Ht.grad.numpy(), rtol=1e-10, atol=1e-14)
    assert np.allclose(out["dW"], Wt.grad.numpy(), rtol=1e-10, atol=1e-14)
    # and central differences of the oracle's own scalar objective
    eps = 1e-6
    rng = np.random.default_rng(0)
    for _ in range(10):
        v, h = rng.integers(0, 12), rng.integers(0, 6)
        Wp, Wm = b["W"].copy(), b["W"].copy()
        Wp[v, h] += eps
        Wm[v, h] -= eps
        fd = (grpo.objective_value(b["hidden"], Wp, *args, **kw) -
              grpo.objective_value(b["hidden"], Wm, *args, **kw)) / (2 * eps)
        assert abs(fd - out["dW"][v, h]) < 1e-8


@pytest.mark.parametrize("kind", [grpo.KL_LOG_RATIO, grpo.KL_NONNEG])
def test_prop1_holds_for_the_token_loss_with_kl(kind):
    # the estimator weights the whole token loss S - beta KL (Eq. 4 inside Eq. 6 / Eq. 9)
    b = _with_ref(tiny_batch(24, [4, 4]), 3, 0.4, kind)
    ft = drivers.full_token(b)
    base = drivers.full_token({k: v for k, v in b.items() if k not in ("ref_logp", "beta_kl", "kl_kind")})
    assert abs(ft["loss"] - base["loss"]) > 1e-3                         # the KL term is really in there
    for e in (drivers.enumerate_urs(b, 0.5), drivers.enumerate_rpc(b, C=1)):
        assert abs(e["prob"] - 1) < 1e-12
        assert abs(e["loss"] - ft["loss"]) < 1e-12
        assert np.abs(e["dW"] - ft["dW"]).max() < 1e-12 and np.abs(e["dH"] - ft["dH"]).max() < 1e-12


# ---------------------------------------------------------------- forward pass alone

def test_forward_logp_is_the_library_log_softmax_and_matches_the_loss_path():
    b = tiny_batch(12, [6, 5])
    f = grpo.forward_logp(b["hidden"], b["W"], b["ids"])
    ref = torch.log_softmax(torch.tensor(b["hidden"]) @ torch.tensor(b["W"]).T, dim=1)
    assert np.allclose(f["logp"], ref[torch.arange(11), torch.tensor(b["ids"])].numpy(), rtol=1e-13)
    assert np.allclose(f["entropy"], -(ref.exp() * ref).sum(1).numpy(), rtol=1e-13)
    out = grpo.loss_and_grads(b["hidden"], b["W"], b["ids"], b["old_logp"], np.ones(11), np.ones(11))
    assert np.array_equal(out["logp"], f["logp"]) and np.array_equal(out["entropy"], f["entropy"])
    e = grpo.forward_logp(np.zeros((0, 8)), b["W"], [])
    assert e["logp"].shape == (0,)
