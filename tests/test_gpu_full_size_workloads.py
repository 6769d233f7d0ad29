"""The remaining workloads at their full size and in the benchmark's launch configuration: the whole
path on the device, then log-probs and dH rows of sampled kept tokens against the oracle (fp64, token
by token) and the selection counts against the oracle's selection of the whole batch."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import synth_inputs as si
from oracle import grpo as ogrpo
from oracle import select as osel
from nat_testlib import DEV, behaviour_logp_from_forward, dh_residual_error, max_rel_err

TOL_BF16 = 2e-2

CASES = [
    ("qwen3_0p6b_head", "urs", dict(p=0.5)),
    ("qwen3_8b_long_cot", "urs", dict(p=0.25)),
    ("wide_head_stress", "mixed", dict(p=0.5, trunc_frac=0.5)),
    ("qwen2p5_math_7b_head", "rpc_drop", dict(min_cut=100)),
]


@pytest.mark.parametrize("name,mode,kw", CASES)
def test_full_size_workload_sampled_tokens(name, mode, kw):
    import paper_2603_06619_amd as nat
    from paper_2603_06619_amd.stage import LossStage
    stage = LossStage(DEV)
    seed = 1000 * si.WORKLOAD_ORDER.index(name)
    b = si.make_batch_torch(name, seed, DEV)
    B, N, G = b["B"], b["N"], b["G"]
    old_logp = behaviour_logp_from_forward(stage, b)
    cu = torch.from_numpy(b["cu_seqlens"]).to(DEV)
    adv = stage.advantage(torch.from_numpy(b["rewards"].reshape(-1)).to(DEV), b["P"], G)
    adv_ref = ogrpo.advantages(b["rewards"]).reshape(-1)
    spr = drop = None
    if mode == "urs":
        scheme = nat.URS
    elif mode == "mixed":
        scheme = nat.URS
        spr = np.array([osel.URS if (i // G) % 2 == 0 else osel.DET for i in range(B)], dtype=np.int32)
    else:
        scheme = nat.RPC
        drop = adv_ref
    params = nat.SelectParams(scheme, seed=seed, step=1, **kw,
                              scheme_per_rollout=None if spr is None else torch.from_numpy(spr).to(DEV),
                              drop_zero_adv=None if drop is None else adv)
    sc = stage.select_compact(params, cu, B, N, hidden=b["hidden"], ids=b["ids"], old_logp=old_logp)
    nk = sc["n_kept"]
    out = stage.loss(sc["hidden_k"], b["W"], sc["ids_k"], sc["old_logp_k"], adv, sc["kept_seq"], sc["kept_w"], nk)
    torch.cuda.synchronize()
    # the oracle's selection of the same batch
    o = osel.select(b["cu_seqlens"], {"urs": osel.URS, "mixed": osel.URS, "rpc_drop": osel.RPC}[mode],
                    p=kw.get("p", 1.0), C=kw.get("min_cut", 1), beta=kw.get("trunc_frac", 1.0), seed=seed, step=1,
                    scheme_per_rollout=spr, drop_zero_adv=drop)
    kept_ref = np.nonzero(o["mask"])[0]
    assert nk == len(kept_ref)
    assert np.array_equal(sc["kept_idx"][:nk].cpu().numpy(), kept_ref)
    # sampled kept tokens through the oracle
    rng = np.random.default_rng(3)
    sample = np.unique(np.concatenate([[0, nk - 1, min(16383, nk - 1), min(16384, nk - 1), min(32767, nk - 1), min(32768, nk - 1)], rng.integers(0, nk, 12)]))
    sidx = torch.from_numpy(sample).to(DEV)
    ref = ogrpo.loss_and_grads(sc["hidden_k"][sidx].float().cpu().numpy(), b["W"].float().cpu().numpy(),
                               sc["ids_k"][sidx].cpu().numpy(), sc["old_logp_k"][sidx].cpu().numpy(),
                               adv_ref[sc["kept_seq"][sidx].cpu().numpy()],
                               sc["kept_w"][sidx].cpu().numpy().astype(np.float64))
    logp = out["logp"][sidx].cpu().numpy()
    assert np.abs(logp - ref["logp"]).max() <= 1e-4
    dH = out["dH"][sidx].float().cpu().numpy()
    for j in range(len(sample)):
        den = np.abs(ref["dH"][j]).max()
        if den > 0:
            assert np.abs(dH[j] - ref["dH"][j]).max() <= TOL_BF16 * den, (name, int(sample[j]))
    res_err, _ = dh_residual_error(dH, ref, b["W"].float().cpu().numpy(), sc["ids_k"][sidx].cpu().numpy(), 2.0 ** -7)
    assert res_err <= TOL_BF16, (name, "dH without the one-hot term", res_err)
    assert np.isfinite(out["loss"].item()) and torch.isfinite(out["dW"]).all()
    print(name, mode, "kept", nk, "of", N, "sampled rel err logp %.2e dH %.2e" %
          (max_rel_err(logp, ref["logp"]), max_rel_err(dH, ref["dH"])))
