"""GPU parity of nat_loss_fwd_bwd_kl against the fp64 oracle: token loss S - beta KL
(Eq. 4, sampled-token forms of its footnote) and the per-token entropy accumulated
in the vocabulary sweep.

Tolerances (max-norm relative error per tensor): loss / logp / dH / dW as for
nat_loss_fwd_bwd (fp32 path 1e-5, bf16 path 2e-2).  KL and entropy are computed
from fp32 accumulators on both paths (no bf16 rounding enters them): 1e-5 on the
fp32 path, 1e-4 on the bf16 path (fast exponential, 1188 partial sums).  The KL
value additionally gets an absolute allowance of 2e-6: it is a function of the fp32
log-prob (|logp| <= 13, so its rounding alone is 8e-7, passed on with slope
|dKL/dlogp| <= 1 here) and the non-negative form exp(d) - d - 1 cancels to ~d^2/2,
three roundings at magnitude <= 2; a lone token with a small d has nothing larger
to be relative to."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import grpo as ogrpo
from nat_testlib import DEV, hip_loss, make_loss_case, max_rel_err, oracle_loss, to_dev
from test_gpu_loss import check, TOL_BF16, TOL_F32

KINDS = [ogrpo.KL_LOG_RATIO, ogrpo.KL_NONNEG]


@pytest.fixture(scope="module")
def stage():
    from paper_2603_06619_amd.stage import LossStage
    return LossStage(DEV)


def add_ref(case, seed, spread=0.3):
    logp = ogrpo.token_logp(case["hidden"], case["W"], case["ids"])
    case["ref_logp"] = (logp + np.random.default_rng(seed).standard_normal(len(logp)) * spread).astype(np.float32)
    return case


def run_both(stage, case, dtype, beta, kind, **kw):
    ref_lp = case.pop("ref_logp")
    ref = oracle_loss(**case, ref_logp=ref_lp, beta_kl=beta, kl_kind=kind, **kw)
    out = hip_loss(stage, case, dtype, ref_logp_k=to_dev(ref_lp), beta_kl=beta, kl_kind=kind, want_kl=True,
                   want_entropy=True, **kw)
    case["ref_logp"] = ref_lp
    return out, ref


def check_diag(out, ref, n, tol):
    kl = out["kl"].cpu().numpy()[:n].astype(np.float64)
    e_kl = float(np.abs(kl - ref["kl"]).max())
    e_h = max_rel_err(out["entropy"].cpu().numpy()[:n], ref["entropy"])
    assert e_kl <= tol * float(np.abs(ref["kl"]).max()) + 2e-6, ("kl", e_kl)
    assert e_h <= tol, ("entropy", e_h)
    return e_kl, e_h


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("n_tok,H,V", [(160, 64, 512), (1, 64, 512), (37, 48, 300)])
def test_fp32_path_with_kl_and_entropy(stage, kind, n_tok, H, V):
    case = add_ref(make_loss_case(40 + n_tok, n_tok, H, V, "f32", noise=0.15), 1)
    out, ref = run_both(stage, case, "f32", 0.3, kind)
    check(out, ref, n_tok, TOL_F32, case)
    check_diag(out, ref, n_tok, 1e-5)


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("n_tok,H,V", [(300, 128, 1000), (700, 256, 5000), (1, 64, 130)])
def test_bf16_path_with_kl_and_entropy(stage, kind, n_tok, H, V):
    case = add_ref(make_loss_case(140 + n_tok, n_tok, H, V, "bf16", noise=0.15, w_std=0.1), 2)
    out, ref = run_both(stage, case, "bf16", 0.25, kind, grad_scale=2.0)
    check(out, ref, n_tok, TOL_BF16, case)
    check_diag(out, ref, n_tok, 1e-4)
    # the KL term is not a rounding-level effect here: without it the gradient differs visibly
    base = oracle_loss(**{k: v for k, v in case.items() if k != "ref_logp"}, grad_scale=2.0)
    assert n_tok < 10 or max_rel_err(base["dW"], ref["dW"]) > 0.05


def test_bf16_entropy_of_peaked_and_flat_policies(stage):
    # half the tokens have a dominant logit (entropy near 0), the others a spread of +-20
    n_tok, H, V = 400, 128, 2000
    case = make_loss_case(33, n_tok, H, V, "bf16", noise=0.1, w_std=0.5)
    Z = case["hidden"].astype(np.float64) @ case["W"].astype(np.float64).T
    ids = case["ids"].copy()
    ids[::2] = Z[::2].argmax(axis=1)
    case["ids"] = ids.astype(np.int32)
    logp = ogrpo.token_logp(case["hidden"], case["W"], case["ids"])
    case["old_logp"] = (logp + np.random.default_rng(5).standard_normal(n_tok) * 0.1).astype(np.float32)
    out, ref = run_both(stage, add_ref(case, 3), "bf16", 0.1, ogrpo.KL_NONNEG)
    check(out, ref, n_tok, TOL_BF16, case)
    check_diag(out, ref, n_tok, 1e-4)
    assert ref["entropy"].min() < 0.5 and ref["entropy"].max() > 2.0
    # flat policy: a zero head gives the uniform distribution, entropy ln V
    case["W"] = np.zeros_like(case["W"])
    case["old_logp"] = np.full(n_tok, -np.log(V), dtype=np.float32)
    out = hip_loss(stage, {k: v for k, v in case.items() if k != "ref_logp"}, "bf16", want_entropy=True)
    assert np.allclose(out["entropy"].cpu().numpy()[:n_tok], np.log(V), rtol=1e-6)


def test_beta_zero_and_diagnostics_leave_the_result_bits_unchanged(stage):
    case = make_loss_case(9, 500, 128, 3000, "bf16", noise=0.1, w_std=0.1)
    a = {k: (v.clone() if v is not None else None) for k, v in hip_loss(stage, case, "bf16").items()}
    ref_lp = to_dev(case["old_logp"] - 0.5)
    b = hip_loss(stage, case, "bf16", ref_logp_k=ref_lp, beta_kl=0.0, kl_kind=1, want_kl=True, want_entropy=True)
    for k in ("loss", "logp", "dH", "dW"):
        assert torch.equal(a[k], b[k]), k
    assert not b["kl"][:500].any()


@pytest.mark.parametrize("kind", KINDS)
def test_bf16_multiple_chunks_with_kl(stage, kind):
    import paper_2603_06619_amd as nat
    n_tok, H, V = 600, 128, 3000
    case = add_ref(make_loss_case(8, n_tok, H, V, "bf16", noise=0.1, w_std=0.1), 4)
    ws_min = nat.loss_workspace_min_bytes(n_tok, H, V, nat.DTYPE_BF16)       # 256-token chunks -> 3 chunks
    out, ref = run_both(stage, case, "bf16", 0.5, kind)
    out_c = hip_loss(stage, {k: v for k, v in case.items() if k != "ref_logp"}, "bf16",
                     ref_logp_k=to_dev(case["ref_logp"]), beta_kl=0.5, kl_kind=kind, want_kl=True, want_entropy=True,
                     ws_bytes=ws_min)
    check(out_c, ref, n_tok, TOL_BF16, case)
    check_diag(out_c, ref, n_tok, 1e-4)


def test_bf16_qwen3_8b_head_reduced_batch_with_kl_and_entropy(stage):
    case = add_ref(make_loss_case(22, 130, 4096, 151936, "bf16"), 5, spread=0.1)
    out, ref = run_both(stage, case, "bf16", 0.04, ogrpo.KL_NONNEG)
    errs = check(out, ref, 130, TOL_BF16, case, label="qwen3-8B head with KL")
    diag = check_diag(out, ref, 130, 1e-4)
    print("qwen3-8B head reduced batch with KL: rel err logp/dH/dW =", errs, " kl/entropy =", diag)
