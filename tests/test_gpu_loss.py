"""GPU parity of nat_loss_fwd_bwd against the fp64 oracle (Eq. 1, 3, 5, 6/9; App. A).

Tolerances (max-norm relative error ||gpu - oracle||_inf / ||oracle||_inf per tensor):
fp32 path <= 1e-5, bf16 path <= 2e-2."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from nat_testlib import DEV, hip_loss, make_loss_case, max_rel_err, oracle_loss, to_dev

TOL_F32 = 1e-5
TOL_BF16 = 2e-2


@pytest.fixture(scope="module")
def stage():
    from paper_2603_06619_amd.stage import LossStage
    return LossStage(DEV)


def check(out, ref, n, tol, dh_dtype_tol=None):
    assert abs(out["loss"].item() - ref["loss"]) <= tol * abs(ref["loss"]) + 1e-12
    e_logp = max_rel_err(out["logp"].cpu().numpy()[:n], ref["logp"])
    e_dh = max_rel_err(out["dH"].float().cpu().numpy()[:n], ref["dH"])
    e_dw = max_rel_err(out["dW"].cpu().numpy(), ref["dW"])
    assert e_logp <= tol, ("logp", e_logp)
    assert e_dh <= tol, ("dH", e_dh)
    assert e_dw <= tol, ("dW", e_dw)
    return e_logp, e_dh, e_dw


@pytest.mark.parametrize("n_tok,H,V", [(160, 64, 512), (1, 64, 512), (37, 48, 300), (300, 64, 512)])
def test_fp32_path(stage, n_tok, H, V):
    case = make_loss_case(10 + n_tok, n_tok, H, V, "f32", noise=0.15)
    ref = oracle_loss(**case)
    out = hip_loss(stage, case, "f32")
    check(out, ref, n_tok, TOL_F32)
    clipped = (ref["r"] > 1.2) | (ref["r"] < 0.8)
    assert n_tok < 30 or clipped.any()


def test_fp32_chunked_workspace_and_accumulate(stage):
    import paper_2603_06619_amd as nat
    case = make_loss_case(5, 50, 64, 512, "f32")
    ref = oracle_loss(**case)
    small = nat.loss_workspace_min_bytes(50, 64, 512, nat.DTYPE_F32) + 6 * 512 * 4     # 7-token chunks
    out = hip_loss(stage, case, "f32", ws_bytes=small)
    check(out, ref, 50, TOL_F32)
    b0 = 2.0 ** -16                    # same magnitude as dW, so fp32 rounding of the sums stays relative
    base = torch.full((512, 64), b0, dtype=torch.float32, device=DEV)
    out2 = hip_loss(stage, case, "f32", dW=base.clone(), accumulate_dw=True)
    assert max_rel_err(out2["dW"].cpu().numpy(), b0 + ref["dW"]) <= TOL_F32


@pytest.mark.parametrize("n_tok,H,V", [
    (300, 128, 1000),        # ragged token tile, vocabulary not a multiple of the granule
    (256, 64, 256),          # exactly one tile
    (700, 256, 5000),        # several tiles each way
    (1, 64, 130),
])
def test_bf16_path_small_shapes(stage, n_tok, H, V):
    case = make_loss_case(100 + n_tok, n_tok, H, V, "bf16", noise=0.15, w_std=0.1)
    ref = oracle_loss(**case)
    out = hip_loss(stage, case, "bf16")
    check(out, ref, n_tok, TOL_BF16)


def test_bf16_grad_scale_and_eps(stage):
    case = make_loss_case(7, 200, 128, 2000, "bf16", noise=0.3, w_std=0.1)
    ref = oracle_loss(**case, eps_lo=0.1, eps_hi=0.28, grad_scale=3.0)
    out = hip_loss(stage, case, "bf16", eps_lo=0.1, eps_hi=0.28, grad_scale=3.0)
    check(out, ref, 200, TOL_BF16)
    assert ((ref["r"] > 1.28) | (ref["r"] < 0.9)).sum() > 10


def test_bf16_peaked_softmax_and_unlikely_targets(stage):
    # logits with a spread of ~ +-20: half the targets are the arg-max (p close to 1, the one-hot
    # term nearly cancels), the rest are random (log(p_max / p_target) up to ~ 40, inside the bound of 70)
    import synth_inputs as si
    from oracle import grpo as ogrpo
    n_tok, H, V = 400, 128, 2000
    case = make_loss_case(31, n_tok, H, V, "bf16", noise=0.1, w_std=0.5)
    Z = case["hidden"].astype(np.float64) @ case["W"].astype(np.float64).T
    ids = case["ids"].copy()
    ids[::2] = Z[::2].argmax(axis=1)
    case["ids"] = ids.astype(np.int32)
    logp = ogrpo.token_logp(case["hidden"], case["W"], case["ids"])
    case["old_logp"] = (logp + np.random.default_rng(5).standard_normal(n_tok) * 0.1).astype(np.float32)
    gap = Z.max(axis=1) - Z[np.arange(n_tok), ids]
    assert gap.max() > 20 and gap.max() < 65 and (np.exp(logp[::2]) > 0.5).sum() > 50
    ref = oracle_loss(**case)
    out = hip_loss(stage, case, "bf16")
    check(out, ref, n_tok, TOL_BF16)


def test_bf16_multiple_chunks_and_accumulate(stage):
    import paper_2603_06619_amd as nat
    n_tok, H, V = 600, 128, 3000
    case = make_loss_case(8, n_tok, H, V, "bf16", noise=0.1, w_std=0.1)
    ref = oracle_loss(**case)
    ws_min = nat.loss_workspace_min_bytes(n_tok, H, V, nat.DTYPE_BF16)       # 256-token chunks -> 3 chunks
    out = hip_loss(stage, case, "bf16", ws_bytes=ws_min)
    check(out, ref, n_tok, TOL_BF16)
    b0 = float(np.abs(ref["dW"]).max())
    base = torch.full((V, H), b0, dtype=torch.float32, device=DEV)
    out2 = hip_loss(stage, case, "bf16", dW=base.clone(), accumulate_dw=True, ws_bytes=ws_min)
    assert max_rel_err(out2["dW"].cpu().numpy() - np.float32(b0), ref["dW"]) <= TOL_BF16


def test_bf16_deterministic_bitwise(stage):
    case = make_loss_case(9, 500, 128, 3000, "bf16", noise=0.1, w_std=0.1)
    a = hip_loss(stage, case, "bf16")
    a = {k: v.clone() for k, v in a.items()}
    b = hip_loss(stage, case, "bf16")
    for k in ("loss", "logp", "dH", "dW"):
        assert torch.equal(a[k], b[k]), k


def test_zero_kept_tokens(stage):
    import paper_2603_06619_amd as nat
    for tdt in (torch.bfloat16, torch.float32):
        W = torch.zeros((512, 64), dtype=tdt, device=DEV)
        dW = torch.full((512, 64), 7.0, dtype=torch.float32, device=DEV)
        loss = torch.full((1,), 3.0, dtype=torch.float32, device=DEV)
        nat.nat_loss_fwd_bwd(None, W, None, None, None, None, None, 0, 0.2, 0.2, 1.0, loss, None, None, dW, False, None)
        torch.cuda.synchronize()
        assert loss.item() == 0.0 and not dW.any()
        dW.fill_(7.0)
        nat.nat_loss_fwd_bwd(None, W, None, None, None, None, None, 0, 0.2, 0.2, 1.0, loss, None, None, dW, True, None)
        torch.cuda.synchronize()
        assert (dW == 7.0).all()


def test_bf16_qwen3_0p6b_head_reduced_batch(stage):
    # full head shape H=1024, V=151936; reduced batch (a few hundred kept tokens)
    case = make_loss_case(21, 300, 1024, 151936, "bf16")
    ref = oracle_loss(**case)
    out = hip_loss(stage, case, "bf16")
    errs = check(out, ref, 300, TOL_BF16)
    print("qwen3-0.6B head reduced batch: rel err logp/dH/dW =", errs)


def test_bf16_qwen3_8b_head_reduced_batch(stage):
    # full head shape H=4096, V=151936; reduced batch
    case = make_loss_case(22, 130, 4096, 151936, "bf16")
    ref = oracle_loss(**case)
    out = hip_loss(stage, case, "bf16")
    errs = check(out, ref, 130, TOL_BF16)
    print("qwen3-8B head reduced batch: rel err logp/dH/dW =", errs)


@pytest.mark.parametrize("H,V,label", [(5120, 151936, "wide head"), (3584, 152064, "Qwen2.5-Math-7B head")])
def test_bf16_other_full_head_shapes_reduced_batch(stage, H, V, label):
    # the remaining head shapes of the workloads: hidden sizes that are 20 and 14 tiles of 256 wide
    case = make_loss_case(23 + H, 150, H, V, "bf16")
    ref = oracle_loss(**case)
    out = hip_loss(stage, case, "bf16")
    errs = check(out, ref, 150, TOL_BF16)
    print(label, "reduced batch: rel err logp/dH/dW =", errs)


def test_bf16_hidden_size_not_a_multiple_of_the_tile(stage):
    # H = 320 (a multiple of 64 but not of 256): the last hidden tile is ragged in dH and dW
    case = make_loss_case(77, 300, 320, 1500, "bf16", noise=0.1, w_std=0.1)
    ref = oracle_loss(**case)
    out = hip_loss(stage, case, "bf16")
    check(out, ref, 300, TOL_BF16)
