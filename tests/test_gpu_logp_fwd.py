"""GPU parity of nat_logp_fwd (forward pass alone) against the fp64 oracle, and its agreement
with the log-probs that nat_loss_fwd_bwd reports for the same tokens."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import grpo as ogrpo
from nat_testlib import DEV, hip_loss, make_loss_case, max_rel_err, to_dev


@pytest.fixture(scope="module")
def stage():
    from paper_2603_06619_amd.stage import LossStage
    return LossStage(DEV)


def run(stage, case, dtype, **kw):
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    n = len(case["ids"])
    out = stage.logp(to_dev(case["hidden"], tdt), to_dev(case["W"], tdt), to_dev(case["ids"]), n, want_entropy=True, **kw)
    torch.cuda.synchronize()
    return out


@pytest.mark.parametrize("n_tok,H,V", [(160, 64, 512), (1, 64, 512), (37, 48, 300)])
def test_fp32_forward(stage, n_tok, H, V):
    case = make_loss_case(60 + n_tok, n_tok, H, V, "f32")
    ref = ogrpo.forward_logp(case["hidden"], case["W"], case["ids"])
    out = run(stage, case, "f32")
    assert max_rel_err(out["logp"].cpu().numpy()[:n_tok], ref["logp"]) <= 1e-5
    assert max_rel_err(out["entropy"].cpu().numpy()[:n_tok], ref["entropy"]) <= 1e-5


@pytest.mark.parametrize("n_tok,H,V", [(300, 128, 1000), (700, 256, 5000), (1, 64, 130), (300, 320, 1500)])
def test_bf16_forward(stage, n_tok, H, V):
    case = make_loss_case(160 + n_tok, n_tok, H, V, "bf16", w_std=0.1)
    ref = ogrpo.forward_logp(case["hidden"], case["W"], case["ids"])
    out = run(stage, case, "bf16")
    # fp32 accumulation of exact bf16 products, nothing is rounded to bf16 on this path
    assert max_rel_err(out["logp"].cpu().numpy()[:n_tok], ref["logp"]) <= 1e-5
    assert max_rel_err(out["entropy"].cpu().numpy()[:n_tok], ref["entropy"]) <= 1e-4


def test_bf16_forward_equals_the_loss_path_bit_for_bit_and_chunks(stage):
    import paper_2603_06619_amd as nat
    n_tok, H, V = 600, 128, 3000
    case = make_loss_case(8, n_tok, H, V, "bf16", w_std=0.1)
    full = hip_loss(stage, case, "bf16", want_entropy=True)
    logp_loss, ent_loss = full["logp"].clone(), full["entropy"].clone()
    out = run(stage, case, "bf16")
    assert torch.equal(out["logp"][:n_tok], logp_loss[:n_tok])
    assert torch.equal(out["entropy"][:n_tok], ent_loss[:n_tok])
    ws_min = nat.logp_workspace_min_bytes(n_tok, H, V, nat.DTYPE_BF16)        # 256-token chunks
    out_c = run(stage, case, "bf16", ws_bytes=ws_min)
    assert torch.equal(out_c["logp"][:n_tok], out["logp"][:n_tok])


def test_bf16_forward_full_head_reduced_batch(stage):
    case = make_loss_case(22, 130, 4096, 151936, "bf16")
    ref = ogrpo.forward_logp(case["hidden"], case["W"], case["ids"])
    out = run(stage, case, "bf16")
    e1 = max_rel_err(out["logp"].cpu().numpy()[:130], ref["logp"])
    e2 = max_rel_err(out["entropy"].cpu().numpy()[:130], ref["entropy"])
    print("forward pass, Qwen3-8B head: rel err logp %.2e entropy %.2e" % (e1, e2))
    assert e1 <= 1e-5 and e2 <= 1e-4


def test_zero_tokens_is_a_no_op(stage):
    import paper_2603_06619_amd as nat
    W = torch.zeros((512, 64), dtype=torch.bfloat16, device=DEV)
    nat.nat_logp_fwd(None, W, None, 0, None, None, None)
