"""GPU parity of nat_advantage / nat_select / nat_compact against the oracle:
bit-exact masks, indices, cut points, offsets and weights (Sec. 3.1, Sec. 4, Eq. 6-9)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import synth_inputs as si
from oracle import grpo as ogrpo
from oracle import select as osel
from nat_testlib import (DEV, assert_select_compact_equal, hip_select_compact, oracle_select_compact, to_dev)


@pytest.fixture(scope="module")
def stage():
    from paper_2603_06619_amd.stage import LossStage
    return LossStage(DEV)


EDGE_LENGTHS = [1, 2, 63, 64, 65, 0, 127, 128, 129, 4095, 4096, 4097, 1, 0, 300]


@pytest.mark.parametrize("scheme,kw", [
    (osel.FULL, {}), (osel.URS, dict(p=0.5)), (osel.URS, dict(p=0.25)), (osel.URS, dict(p=1.0)),
    (osel.URS, dict(p=0.37)), (osel.RPC, dict(C=1)), (osel.RPC, dict(C=100)), (osel.RPC, dict(C=10 ** 6)),
    (osel.DET, dict(beta=0.5)), (osel.DET, dict(beta=1.0))])
def test_edge_lengths_all_schemes(stage, scheme, kw):
    cu = np.concatenate([[0], np.cumsum(EDGE_LENGTHS)]).astype(np.int64)
    for seed in (0, 1, 0xDEADBEEFCAFE):
        o = oracle_select_compact(cu, scheme, seed=seed, step=3, base=17, **kw)
        h = hip_select_compact(stage, cu, scheme, seed=seed, step=3, base=17, **kw)
        assert_select_compact_equal(h, o, int(cu[-1]))


def test_many_seeds_small_batches(stage):
    rng = np.random.default_rng(0)
    for trial in range(60):
        B = int(rng.integers(1, 12))
        T = rng.integers(0, 200, B)
        cu = np.concatenate([[0], np.cumsum(T)]).astype(np.int64)
        scheme = int(rng.integers(0, 4))
        kw = dict(p=float(rng.choice([0.1, 0.5, 0.9])), C=int(rng.choice([1, 5, 50])), beta=float(rng.choice([0.3, 0.5])),
                  seed=int(rng.integers(0, 2 ** 63)), step=int(rng.integers(0, 2 ** 32)), base=int(rng.integers(0, 10 ** 6)))
        o = oracle_select_compact(cu, scheme, n_rollouts=B + 3, **kw)
        h = hip_select_compact(stage, cu, scheme, n_rollouts=B + 3, **kw)
        assert_select_compact_equal(h, o, int(cu[-1]))


def test_mixed_schemes_per_rollout_and_gather(stage):
    lay = si.batch_layout("wide_head_stress", 5, P=6, G=4)
    cu = lay["cu_seqlens"]
    N = lay["N"]
    spr = np.where((np.arange(24) // 4) % 2 == 0, osel.URS, osel.DET).astype(np.int32)
    rng = np.random.default_rng(1)
    hidden = rng.standard_normal((N, 64), dtype=np.float32)
    ids = rng.integers(0, 1000, N).astype(np.int32)
    old = rng.standard_normal(N).astype(np.float32)
    o = oracle_select_compact(cu, osel.URS, p=0.5, beta=0.5, seed=9, spr=spr)
    for tdt in (torch.float32, torch.bfloat16):
        h = hip_select_compact(stage, cu, osel.URS, p=0.5, beta=0.5, seed=9, spr=spr,
                               hidden=to_dev(hidden, tdt), ids=to_dev(ids), old_logp=to_dev(old))
        assert_select_compact_equal(h, o, N)
        nk = o["n_kept"]
        ref_rows = to_dev(hidden, tdt)[torch.from_numpy(o["kept_idx"]).long().to(DEV)]
        assert torch.equal(h["hidden_k"][:nk], ref_rows)
        assert np.array_equal(h["ids_k"].cpu().numpy()[:nk], ids[o["kept_idx"]])
        assert np.array_equal(h["old_logp_k"].cpu().numpy()[:nk], old[o["kept_idx"]])


@pytest.mark.parametrize("name,scheme,kw", [
    ("qwen3_8b_head_rpc", osel.RPC, dict(C=1)),
    ("qwen3_8b_long_cot", osel.URS, dict(p=0.5)),
    ("qwen3_8b_long_cot", osel.RPC, dict(C=100)),
    ("wide_head_stress", osel.DET, dict(beta=0.5))])
def test_full_size_batches_bit_exact(stage, name, scheme, kw):
    lay = si.batch_layout(name, 1000 * si.WORKLOAD_ORDER.index(name))
    cu = lay["cu_seqlens"]
    o = oracle_select_compact(cu, scheme, seed=77, step=1, **kw)
    h = hip_select_compact(stage, cu, scheme, seed=77, step=1, **kw)
    assert_select_compact_equal(h, o, lay["N"])
    if scheme == osel.RPC and kw["C"] == 1:
        # expected retained fraction about one half (Sec. 4, uniform cutoff)
        assert 0.35 < o["n_kept"] / lay["N"] < 0.65


def test_empty_batch_and_all_dropped(stage):
    cu = np.array([0, 0, 0], dtype=np.int64)
    h = hip_select_compact(stage, cu, osel.URS, p=0.5)
    assert h["n_kept"] == 0 and h["cu_kept"].cpu().tolist() == [0, 0, 0]
    cu = np.array([0, 1, 2, 3], dtype=np.int64)          # DET with beta=.5 on length-1 rollouts keeps nothing
    o = oracle_select_compact(cu, osel.DET, beta=0.5)
    h = hip_select_compact(stage, cu, osel.DET, beta=0.5)
    assert o["n_kept"] == 0
    assert_select_compact_equal(h, o, 3)


def test_advantage_matches_eq2(stage):
    rng = np.random.default_rng(3)
    for P, G in [(1, 1), (2, 4), (16, 8), (8, 16), (5, 70), (3, 130)]:
        R = si.draw_rewards(P, G, rng, equal_reward_frac=0.3)
        if G > 8:
            R = R + rng.random((P, G)).astype(np.float32)
            R[0] = 2.0
        adv = stage.advantage(to_dev(R.reshape(-1)), P, G, 1e-6).cpu().numpy().reshape(P, G)
        ref = ogrpo.advantages(R, 1e-6)
        assert np.abs(adv - ref).max() <= 2e-6 * max(1.0, np.abs(ref).max())
        assert (adv[np.ptp(R, axis=1) == 0] == 0).all()       # equal rewards: exactly zero


@pytest.mark.parametrize("scheme,kw", [(osel.FULL, {}), (osel.URS, dict(p=0.5)), (osel.RPC, dict(C=100)),
                                        (osel.DET, dict(beta=0.5))])
def test_zero_advantage_rollouts_are_dropped(stage, scheme, kw):
    # the paper's second model workload: a quarter of the prompts have all-equal rewards; Eq. 2 on the device
    # gives exactly 0 there, and those rollouts keep nothing
    lay = si.batch_layout("qwen2p5_math_7b_head", 5000)
    cu, B, P, G = lay["cu_seqlens"], lay["B"], lay["P"], lay["G"]
    adv_dev = stage.advantage(to_dev(lay["rewards"].reshape(-1)), P, G)
    adv = adv_dev.cpu().numpy()
    adv_ref = ogrpo.advantages(lay["rewards"]).reshape(-1)
    assert np.array_equal(adv == 0, adv_ref == 0) and (adv == 0).sum() >= B // 4
    o = oracle_select_compact(cu, scheme, seed=3, step=2, drop=adv_ref, **kw)
    h = hip_select_compact(stage, cu, scheme, seed=3, step=2, drop=adv, **kw)
    assert_select_compact_equal(h, o, lay["N"])
    full = oracle_select_compact(cu, scheme, seed=3, step=2, **kw)
    assert o["n_kept"] < full["n_kept"]
