"""Selection and compaction on a batch far beyond the workloads (2^26 tokens in 2048 rollouts): properties
that hold at any size on the whole result, and the oracle on sampled rollouts and tokens."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import select as osel
from nat_testlib import DEV, to_dev


@pytest.fixture(scope="module")
def big():
    from paper_2603_06619_amd.stage import LossStage
    rng = np.random.default_rng(12)
    B, N = 2048, 1 << 26
    cuts = np.sort(rng.choice(np.arange(1, N), size=B - 1, replace=False))
    cu = np.concatenate([[0], cuts, [N]]).astype(np.int64)
    cu[700] = cu[699]                                     # an empty rollout in the middle
    return LossStage(DEV), cu, B, N


def _unpack(mask_words, lo, hi):
    w = mask_words[lo // 32:(hi + 31) // 32].cpu().numpy().view(np.uint32)
    bits = np.unpackbits(w.view(np.uint8), bitorder="little")
    return bits[lo - (lo // 32) * 32: lo - (lo // 32) * 32 + (hi - lo)].astype(bool)


@pytest.mark.parametrize("scheme,kw", [(osel.URS, dict(p=0.3)), (osel.RPC, dict(C=50))])
def test_large_batch_properties_and_samples(big, scheme, kw):
    import paper_2603_06619_amd as nat
    stage, cu, B, N = big
    params = nat.SelectParams(scheme, p=kw.get("p", 1.0), min_cut=kw.get("C", 1), seed=99, step=5, rollout_id_base=3)
    sc = stage.select_compact(params, to_dev(cu), B, N, n_rollouts_global=B)
    nk = sc["n_kept"]
    words = sc["mask_bits"]
    # whole-result properties
    pop = int(sum(int(np.unpackbits(words[a:a + (1 << 20)].cpu().numpy().view(np.uint8)).sum())
                  for a in range(0, words.numel(), 1 << 20)))
    assert nk == pop == int(sc["n_kept_dev"].item())
    idx = sc["kept_idx"][:nk]
    assert bool((idx[1:] > idx[:-1]).all()) and int(idx[0]) >= 0 and int(idx[-1]) < N
    cuk = sc["cu_kept"].cpu().numpy()
    assert cuk[0] == 0 and cuk[-1] == nk and (np.diff(cuk) >= 0).all() and cuk[700] == cuk[699]
    seq = sc["kept_seq"][:nk]
    assert bool((seq[1:] >= seq[:-1]).all())
    assert bool((sc["kept_w"][:nk] > 0).all())
    if scheme == osel.RPC:
        cut = sc["cut_len"].cpu().numpy()
        T = np.diff(cu)
        ref_cut = np.array([osel.rpc_cut(int(T[i]), kw["C"], 99, 5, 3 + i) for i in range(B)])
        assert np.array_equal(cut, ref_cut)
        assert np.array_equal(np.diff(cuk), ref_cut)                  # kept tokens are exactly the prefixes
    # sampled rollouts against the oracle, bit for bit
    rng = np.random.default_rng(1)
    for i in np.concatenate([[0, 699, 700, 701, B - 1], rng.integers(0, B, 8)]):
        lo, hi = int(cu[i]), int(cu[i + 1])
        T = hi - lo
        if scheme == osel.URS:
            m = osel.urs_mask(T, kw["p"], 99, 5, 3 + int(i))
        else:
            m = np.arange(1, T + 1) <= osel.rpc_cut(T, kw["C"], 99, 5, 3 + int(i))
        assert np.array_equal(_unpack(words, lo, hi), m), int(i)
        assert cuk[i + 1] - cuk[i] == int(m.sum())
        kept_t = np.nonzero(m)[0][:50] + 1
        if len(kept_t) == 0:
            continue
        w_dev = sc["kept_w"][int(cuk[i]):int(cuk[i]) + len(kept_t)].cpu().numpy()
        w_ref = osel.ht_weights_rollout(scheme, T, kept_t, B, p=kw.get("p", 1.0), C=kw.get("C", 1))
        assert np.array_equal(w_dev.view(np.uint32), w_ref.view(np.uint32)), int(i)
