"""GPU parity of nat_loss_fwd_bwd against the fp64 oracle (Eq. 1, 3, 5, 6/9; App. A).

Tolerances.  Per tensor, max-norm relative error ||gpu - oracle||_inf / ||oracle||_inf:
fp32 path <= 1e-5, bf16 path <= 2e-2 (dH, dW).  Because the one-hot term of dz dominates those
maxima when the soft-max is near-uniform, the two backward contractions are also checked on
their own at the same tolerance: rows of dW that no token targets against the largest such
entry, and dH with the one-hot term removed on both sides against the largest residual entry
(nat_testlib.contraction_errors; the rounding that the full value of an entry carries is allowed on
top, entry by entry: 2^-7 |dH| on the bf16 path, where the one-hot term is rounded to bf16 twice at a
unit roundoff of 2^-8 each, once as the patched numerator and once in the stored output; 2^-18 |dH| on
the fp32 path, whose sequential fp32 sum over V terms carries about sqrt(V) 2^-24 of the full value;
entries where the one-hot term is small are held to the bare tolerance).  Log-probs and the loss come from fp32 accumulators on both
paths and are held to an absolute 1e-4 (log-probs; 1e-5 relative on the fp32 path) and a
relative 1e-4 (loss; 1e-5 on the fp32 path).  Relative Frobenius errors are printed."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from nat_testlib import DEV, contraction_errors, hip_loss, make_loss_case, max_rel_err, oracle_loss, to_dev

TOL_F32 = 1e-5
TOL_BF16 = 2e-2
TOL_LOGP_ABS_BF16 = 1e-4          # fp32 accumulation of exact bf16 products; |logp| ~ 5..13
TOL_LOSS_BF16 = 1e-4


@pytest.fixture(scope="module")
def stage():
    from paper_2603_06619_amd.stage import LossStage
    return LossStage(DEV)


def check(out, ref, n, tol, case=None, logp_atol=None, label=None):
    """Whole-tensor bounds, and (given the case's inputs) the contraction-only bounds."""
    bf16 = tol == TOL_BF16
    tol_loss = TOL_LOSS_BF16 if bf16 else tol
    e_loss = abs(out["loss"].item() - ref["loss"]) / max(abs(ref["loss"]), 1e-300)
    assert e_loss <= tol_loss + 1e-12, ("loss", e_loss)
    logp = out["logp"].cpu().numpy()[:n].astype(np.float64)
    a_logp = float(np.abs(logp - ref["logp"]).max())
    if bf16:
        assert a_logp <= (TOL_LOGP_ABS_BF16 if logp_atol is None else logp_atol), ("logp abs", a_logp)
    e_logp = max_rel_err(logp, ref["logp"])
    dH = out["dH"].float().cpu().numpy()[:n]
    dW = out["dW"].cpu().numpy()
    e_dh = max_rel_err(dH, ref["dH"])
    e_dw = max_rel_err(dW, ref["dW"])
    assert e_logp <= (tol if not bf16 else 1e-4), ("logp", e_logp)
    assert e_dh <= tol, ("dH", e_dh)
    assert e_dw <= tol, ("dW", e_dw)
    if case is not None:
        ce = contraction_errors(dH, dW, ref, case["hidden"], case["W"], case["ids"], 2.0 ** -7 if bf16 else 2.0 ** -18)
        print("%s: loss %.1e logp abs %.1e | dH max %.1e fro %.1e residual %.1e (residual is %.1e of max) | "
              "dW max %.1e fro %.1e off-target rows %.1e (%.1e of max)"
              % (label or "case", e_loss, a_logp, e_dh, ce["dH_fro"], ce["dH_res"], ce["dH_res_share"], e_dw,
                 ce["dW_fro"], ce["dW_off"], ce["dW_off_share"]))
        assert ce["dH_res"] <= tol, ("dH without the one-hot term", ce)
        assert ce["dW_off"] <= tol, ("off-target rows of dW", ce)
    return e_logp, e_dh, e_dw


@pytest.mark.parametrize("n_tok,H,V", [(160, 64, 512), (1, 64, 512), (37, 48, 300), (300, 64, 512)])
def test_fp32_path(stage, n_tok, H, V):
    case = make_loss_case(10 + n_tok, n_tok, H, V, "f32", noise=0.15)
    ref = oracle_loss(**case)
    out = hip_loss(stage, case, "f32")
    check(out, ref, n_tok, TOL_F32, case)
    clipped = (ref["r"] > 1.2) | (ref["r"] < 0.8)
    assert n_tok < 30 or clipped.any()


def test_fp32_chunked_workspace_and_accumulate(stage):
    import paper_2603_06619_amd as nat
    case = make_loss_case(5, 50, 64, 512, "f32")
    ref = oracle_loss(**case)
    small = nat.loss_workspace_min_bytes(50, 64, 512, nat.DTYPE_F32) + 6 * 512 * 4     # 7-token chunks
    out = hip_loss(stage, case, "f32", ws_bytes=small)
    check(out, ref, 50, TOL_F32, case)
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
    check(out, ref, n_tok, TOL_BF16, case)


def test_bf16_grad_scale_and_eps(stage):
    case = make_loss_case(7, 200, 128, 2000, "bf16", noise=0.3, w_std=0.1)
    ref = oracle_loss(**case, eps_lo=0.1, eps_hi=0.28, grad_scale=3.0)
    out = hip_loss(stage, case, "bf16", eps_lo=0.1, eps_hi=0.28, grad_scale=3.0)
    check(out, ref, 200, TOL_BF16, case)
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
    check(out, ref, n_tok, TOL_BF16, case)


def test_bf16_multiple_chunks_and_accumulate(stage):
    import paper_2603_06619_amd as nat
    n_tok, H, V = 600, 128, 3000
    case = make_loss_case(8, n_tok, H, V, "bf16", noise=0.1, w_std=0.1)
    ref = oracle_loss(**case)
    ws_min = nat.loss_workspace_min_bytes(n_tok, H, V, nat.DTYPE_BF16)       # 256-token chunks -> 3 chunks
    out = hip_loss(stage, case, "bf16", ws_bytes=ws_min)
    check(out, ref, n_tok, TOL_BF16, case)
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
    errs = check(out, ref, 300, TOL_BF16, case, label="qwen3-0.6B head")
    print("qwen3-0.6B head reduced batch: rel err logp/dH/dW =", errs)


def test_bf16_qwen3_8b_head_reduced_batch(stage):
    # full head shape H=4096, V=151936; reduced batch
    case = make_loss_case(22, 130, 4096, 151936, "bf16")
    ref = oracle_loss(**case)
    out = hip_loss(stage, case, "bf16")
    errs = check(out, ref, 130, TOL_BF16, case, label="qwen3-8B head")
    print("qwen3-8B head reduced batch: rel err logp/dH/dW =", errs)


@pytest.mark.parametrize("H,V,label", [(5120, 151936, "wide head"), (3584, 152064, "Qwen2.5-Math-7B head")])
def test_bf16_other_full_head_shapes_reduced_batch(stage, H, V, label):
    # the remaining head shapes of the workloads: hidden sizes that are 20 and 14 tiles of 256 wide
    case = make_loss_case(23 + H, 150, H, V, "bf16")
    ref = oracle_loss(**case)
    out = hip_loss(stage, case, "bf16")
    errs = check(out, ref, 150, TOL_BF16, case, label=label)
    print(label, "reduced batch: rel err logp/dH/dW =", errs)


def test_bf16_hidden_size_not_a_multiple_of_the_tile(stage):
    # H = 320 (a multiple of 64 but not of 256): the last hidden tile is ragged in dH and dW
    case = make_loss_case(77, 300, 320, 1500, "bf16", noise=0.1, w_std=0.1)
    ref = oracle_loss(**case)
    out = hip_loss(stage, case, "bf16")
    check(out, ref, 300, TOL_BF16, case)


def test_bf16_dw_leftover_tiles_cut_into_token_ranges(stage):
    # 8 dW tiles on 256 compute units: all of them are "left over" after the last full round, so the library
    # cuts their token axis (8173 tokens = 256 k-slices) into 8 ranges and adds the partial tiles in range
    # order; checked against the oracle element by element, with and without accumulation, and bit for bit
    # between two runs
    n_tok, H, V = 8192 - 19, 256, 2048
    case = make_loss_case(55, n_tok, H, V, "bf16", noise=0.1, w_std=0.1)
    ref = oracle_loss(**case)
    out = hip_loss(stage, case, "bf16")
    check(out, ref, n_tok, TOL_BF16, case, label="dW tiles in 8 token ranges")
    first = out["dW"].clone()
    b0 = float(np.abs(ref["dW"]).max())
    base = torch.full((V, H), b0, dtype=torch.float32, device=DEV)
    out2 = hip_loss(stage, case, "bf16", dW=base.clone(), accumulate_dw=True)
    assert max_rel_err(out2["dW"].cpu().numpy() - np.float32(b0), ref["dW"]) <= TOL_BF16
    again = hip_loss(stage, case, "bf16")
    assert torch.equal(first, again["dW"])


def test_bf16_full_vocabulary_mid_size_every_element_of_dw(stage):
    # the whole vocabulary (V = 151936, H = 1024) with enough tokens for 9 token tiles, and a workspace
    # that forces 3 chunks: dW (and everything else) against the oracle element by element
    import paper_2603_06619_amd as nat
    n_tok, H, V = 2304 - 37, 1024, 151936                  # ragged last token tile
    case = make_loss_case(301, n_tok, H, V, "bf16")
    ref = oracle_loss(**case)
    ws = nat.loss_workspace_bytes(768, H, V, nat.DTYPE_BF16) + 64 * 1024     # room for 768-token chunks, not 1024
    assert ws < nat.loss_workspace_bytes(1024, H, V, nat.DTYPE_BF16)
    out = hip_loss(stage, case, "bf16", ws_bytes=ws)
    check(out, ref, n_tok, TOL_BF16, case, label="full vocabulary, H = 1024, %d tokens in 3 chunks" % n_tok)
    # one chunk gives the same log-probs bit for bit and dW within rounding of the chunked sum (with one chunk
    # the 72 dW tiles left over after 9 full rounds are cut into two token ranges)
    one = hip_loss(stage, case, "bf16")
    assert torch.equal(one["logp"][:n_tok], out["logp"][:n_tok])
    check(one, ref, n_tok, TOL_BF16, case, label="same, one chunk")
