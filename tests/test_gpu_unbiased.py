"""Prop. 1 on the device: the mean of the HIP path's estimate over many seeded masks converges
to the full-token GRPO loss and gradient (URS, RPC, a general cut schedule), and deterministic
truncation does not (the biased control of Sec. 4).  The full-token reference is the oracle's."""
import math

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import synth_inputs as si
from oracle import drivers as odrv
from oracle import grpo as ogrpo
from nat_testlib import DEV, to_dev


@pytest.fixture(scope="module")
def setup():
    import paper_2603_06619_amd as nat
    from paper_2603_06619_amd.stage import LossStage
    b = si.make_batch_numpy("tiny_fp32", 77, P=2, G=3, lengths=("uniform", 5, 12), H=16, V=32)
    old = (ogrpo.token_logp(b["hidden"], b["W"], b["ids"]) + 3.0 * b["logp_noise"]).astype(np.float32)
    adv = ogrpo.advantages(b["rewards"]).reshape(-1)
    if not adv.any():                                    # make sure some rollout has a non-zero advantage
        adv = np.linspace(-1, 1, b["B"])
    batch = dict(cu_seqlens=b["cu_seqlens"], hidden=b["hidden"].astype(np.float64), W=b["W"].astype(np.float64),
                 ids=b["ids"], old_logp=old.astype(np.float64), adv=adv.astype(np.float64))
    ft = odrv.full_token(batch)
    dev = dict(cu=to_dev(b["cu_seqlens"]), hidden=to_dev(b["hidden"]), W=to_dev(b["W"]), ids=to_dev(b["ids"]),
               old=to_dev(old), adv=to_dev(adv.astype(np.float32)))
    return nat, LossStage(DEV), b, dev, ft


def _mean_estimate(nat, stage, b, dev, K, make_params, **sel_kw):
    V, H = b["W"].shape
    s1 = np.zeros(1 + V * H)
    s2 = np.zeros(1 + V * H)
    for seed in range(K):
        sc = stage.select_compact(make_params(seed), dev["cu"], b["B"], b["N"], hidden=dev["hidden"], ids=dev["ids"],
                                  old_logp=dev["old"], **sel_kw)
        out = stage.loss(sc["hidden_k"], dev["W"], sc["ids_k"], sc["old_logp_k"], dev["adv"], sc["kept_seq"],
                         sc["kept_w"], sc["n_kept"])
        v = np.concatenate([out["loss"].cpu().numpy().astype(np.float64), out["dW"].cpu().numpy().ravel().astype(np.float64)])
        s1 += v
        s2 += v * v
    mean = s1 / K
    std = np.sqrt(np.maximum(s2 / K - mean ** 2, 0))
    return mean, std


@pytest.mark.parametrize("which", ["urs", "rpc", "rpc_min_cut", "schedule", "poisson"])
def test_mean_over_seeds_converges_to_full_token(setup, which):
    nat, stage, b, dev, ft = setup
    K = 1500
    kw = {}
    if which == "urs":
        mk = lambda s: nat.SelectParams(nat.URS, p=0.5, seed=1000 + s)
    elif which == "rpc":
        mk = lambda s: nat.SelectParams(nat.RPC, min_cut=1, seed=2000 + s)
    elif which == "rpc_min_cut":
        mk = lambda s: nat.SelectParams(nat.RPC, min_cut=4, seed=3000 + s)
    elif which == "schedule":
        w = si.draw_schedule_weights(b["lengths"], "tail_mass", seed=1)
        kw = dict(schedule_weights=to_dev(w.view(np.int32)))
        mk = lambda s: nat.SelectParams(nat.FULL, seed=4000 + s)
    else:
        kw = dict(poisson_pi=to_dev(si.draw_inclusion_probs(b["N"], seed=2, floor=0.3)))
        mk = lambda s: nat.SelectParams(nat.FULL, seed=5000 + s)
    mean, std = _mean_estimate(nat, stage, b, dev, K, mk, **kw)
    ref = np.concatenate([[ft["loss"]], ft["dW"].ravel()])
    tol = 5 * std / math.sqrt(K) + 1e-5 * np.abs(ref).max()      # sampling error + the fp32 path's rounding
    assert (np.abs(mean - ref) <= tol).all(), float((np.abs(mean - ref) / tol).max())
    assert std.max() > 0                                          # the masks really vary with the seed


def test_deterministic_truncation_is_biased_on_the_device(setup):
    nat, stage, b, dev, ft = setup
    mean, std = _mean_estimate(nat, stage, b, dev, 3, lambda s: nat.SelectParams(nat.DET, trunc_frac=0.5, seed=s))
    assert std.max() < 1e-9                                       # no randomness at all
    ref = ft["dW"].ravel()
    assert np.abs(mean[1:] - ref).max() > 1e-2 * np.abs(ref).max()
