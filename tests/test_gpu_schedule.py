"""GPU parity of nat_select_schedule / nat_select_poisson / nat_compact_pi /
nat_prefix_pack against the oracle: bit-exact cuts, masks, survival
probabilities, indices, weights and packing (Sec. 3.1, Sec. 4 Eq. 7-9)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import synth_inputs as si
from oracle import schedule as osch
from oracle import select as osel
from oracle import drivers as odrv
from nat_testlib import DEV, make_loss_case, max_rel_err, to_dev


@pytest.fixture(scope="module")
def stage():
    from paper_2603_06619_amd.stage import LossStage
    return LossStage(DEV)


def _params(seed=0, step=0, base=0):
    import paper_2603_06619_amd as nat
    return nat.SelectParams(nat.FULL, seed=seed, step=step, rollout_id_base=base)


def _check_compact(h, o, check_w=True):
    nk = o["n_kept"]
    assert h["n_kept"] == nk
    assert np.array_equal(h["kept_idx"].cpu().numpy()[:nk], o["kept_idx"])
    assert np.array_equal(h["kept_seq"].cpu().numpy()[:nk], o["kept_seq"])
    assert np.array_equal(h["cu_kept"].cpu().numpy(), o["cu_kept"])
    if check_w:
        assert np.array_equal(h["kept_w"].cpu().numpy()[:nk].view(np.uint32), o["kept_w"].view(np.uint32))


def _mask_words(h, mask):
    ref = osel.pack_mask_bits(mask)
    return np.array_equal(h["mask_bits"].cpu().numpy().view(np.uint32)[:len(ref)], ref)


EDGE_LENGTHS = [1, 2, 255, 256, 257, 0, 511, 513, 4097, 1, 0, 300, 9000]


@pytest.mark.parametrize("kind", ["uniform", "min_cut", "tail_mass", "random", "sparse"])
def test_schedule_edge_lengths_bit_exact(stage, kind):
    cu = np.concatenate([[0], np.cumsum(EDGE_LENGTHS)]).astype(np.int64)
    B, N = len(EDGE_LENGTHS), int(cu[-1])
    w = si.draw_schedule_weights(EDGE_LENGTHS, kind, seed=3)
    if kind == "random":
        w[cu[2]:cu[3]] = 0                                        # one rollout without a schedule
        w[cu[7]:cu[8]] = 2 ** 32 - 1                              # and one of maximal weights
    for seed in (0, 5, 0xFEEDFACE12345):
        o = osch.select_schedule(cu, w, seed=seed, step=2, rollout_id_base=11)
        oc = osch.compact_pi(o["mask"], o["pi"], cu, B + 2)
        h = stage.select_compact(_params(seed, 2, 11), to_dev(cu), B, N, B + 2,
                                 schedule_weights=to_dev(w.view(np.int32)))
        assert np.array_equal(h["cut_len"].cpu().numpy(), o["cut_len"])
        assert _mask_words(h, o["mask"])
        assert np.array_equal(h["pi"].cpu().numpy()[:N].view(np.uint64), o["pi"].view(np.uint64))
        _check_compact(h, oc)


def test_schedule_full_size_batch_and_gather(stage):
    lay = si.batch_layout("qwen3_8b_head_rpc", 2000)
    cu, B, N = lay["cu_seqlens"], lay["B"], lay["N"]
    w = si.draw_schedule_weights(lay["lengths"], "tail_mass", seed=1)
    o = osch.select_schedule(cu, w, seed=77, step=1)
    oc = osch.compact_pi(o["mask"], o["pi"], cu, B)
    ids = np.random.default_rng(0).integers(0, 151936, N).astype(np.int32)
    h = stage.select_compact(_params(77, 1), to_dev(cu), B, N, B, ids=to_dev(ids),
                             schedule_weights=to_dev(w.view(np.int32)))
    assert np.array_equal(h["cut_len"].cpu().numpy(), o["cut_len"])
    assert _mask_words(h, o["mask"])
    assert np.array_equal(h["pi"].cpu().numpy()[:N].view(np.uint64), o["pi"].view(np.uint64))
    _check_compact(h, oc)
    assert np.array_equal(h["ids_k"].cpu().numpy()[:oc["n_kept"]], ids[oc["kept_idx"]])


def test_uniform_schedule_weights_equal_the_uniform_rpc_closed_form(stage):
    # property at any size: all-ones weights give p_t = (T - t + 1)/T on the device as well
    lay = si.batch_layout("qwen3_8b_long_cot", 3000, P=4, G=4)
    cu, B, N = lay["cu_seqlens"], lay["B"], lay["N"]
    w = si.draw_schedule_weights(lay["lengths"], "uniform", seed=0)
    h = stage.select_compact(_params(1, 0), to_dev(cu), B, N, B, schedule_weights=to_dev(w.view(np.int32)))
    pi = h["pi"].cpu().numpy()[:N]
    ref = np.concatenate([osel.inclusion_prob(osel.RPC, int(T), C=1) for T in lay["lengths"]])
    assert np.array_equal(pi, ref)
    cut = h["cut_len"].cpu().numpy()
    assert (cut >= 1).all() and (cut <= lay["lengths"]).all()


def test_poisson_bit_exact_and_weights(stage):
    rng = np.random.default_rng(4)
    for trial in range(20):
        B = int(rng.integers(1, 10))
        T = rng.integers(0, 400, B)
        cu = np.concatenate([[0], np.cumsum(T)]).astype(np.int64)
        N = int(cu[-1])
        pi = si.draw_inclusion_probs(N, seed=trial)
        pi[rng.random(N) < 0.05] = 0.0                             # never kept
        pi[rng.random(N) < 0.02] = 2.0 ** -40                      # below one part in 2^32: never kept either
        seed, step, base = int(rng.integers(0, 2 ** 63)), int(rng.integers(0, 2 ** 32)), int(rng.integers(0, 1000))
        m = osch.select_poisson(cu, pi, seed=seed, step=step, rollout_id_base=base)
        oc = osch.compact_pi(m, pi, cu, B)
        h = stage.select_compact(_params(seed, step, base), to_dev(cu), B, N, B, poisson_pi=to_dev(pi))
        assert _mask_words(h, m)
        _check_compact(h, oc)


def test_poisson_constant_probability_reproduces_urs_on_device(stage):
    import paper_2603_06619_amd as nat
    lay = si.batch_layout("qwen3_0p6b_head", 1000)
    cu, B, N = to_dev(lay["cu_seqlens"]), lay["B"], lay["N"]
    for p in (0.25, 0.5, 0.37):
        hp = stage.select_compact(_params(9, 4, 100), cu, B, N, B,
                                  poisson_pi=torch.full((N,), p, dtype=torch.float64, device=DEV))
        hu = stage.select_compact(nat.SelectParams(nat.URS, p=p, seed=9, step=4, rollout_id_base=100), cu, B, N, B)
        assert torch.equal(hp["mask_bits"], hu["mask_bits"])
        assert hp["n_kept"] == hu["n_kept"]
        # weights: 1/((B T) p) against 1/(B T p): at most one fp64 rounding apart before the fp32 rounding
        nk = hp["n_kept"]
        a, b = hp["kept_w"][:nk].cpu().numpy(), hu["kept_w"][:nk].cpu().numpy()
        assert np.abs(a.view(np.int32) - b.view(np.int32)).max() <= 1


def test_poisson_full_size_batch(stage):
    lay = si.batch_layout("qwen3_8b_long_cot", 3000)
    cu, B, N = lay["cu_seqlens"], lay["B"], lay["N"]
    pi = si.draw_inclusion_probs(N, seed=2)
    m = osch.select_poisson(cu, pi, seed=5, step=0)
    h = stage.select_compact(_params(5, 0), to_dev(cu), B, N, B, poisson_pi=to_dev(pi))
    assert _mask_words(h, m)
    # weights of a sample of kept tokens, one by one
    nk = h["n_kept"]
    assert nk == int(m.sum())
    idx = h["kept_idx"].cpu().numpy()[:nk]
    assert np.array_equal(idx, np.nonzero(m)[0])
    seq = h["kept_seq"].cpu().numpy()[:nk]
    wts = h["kept_w"].cpu().numpy()[:nk]
    for k in np.random.default_rng(0).integers(0, nk, 2000):
        assert wts[k] == osch.ht_weight_pi(lay["lengths"][seq[k]], pi[idx[k]], B)


def test_schedule_and_poisson_drop_zero_advantage_rollouts(stage):
    import paper_2603_06619_amd as nat
    lengths = [300, 1, 70, 1030, 0, 64]
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    B, N = len(lengths), int(cu[-1])
    adv = np.array([0.5, 0.0, -1.0, 0.0, 0.0, 2.0], dtype=np.float32)
    params = nat.SelectParams(nat.FULL, seed=8, step=1, drop_zero_adv=to_dev(adv))
    w = si.draw_schedule_weights(lengths, "random", seed=2)
    o = osch.select_schedule(cu, w, seed=8, step=1, drop_zero_adv=adv)
    h = stage.select_compact(params, to_dev(cu), B, N, B, schedule_weights=to_dev(w.view(np.int32)))
    assert np.array_equal(h["cut_len"].cpu().numpy(), o["cut_len"])
    assert _mask_words(h, o["mask"])
    assert np.array_equal(h["pi"].cpu().numpy()[:N].view(np.uint64), o["pi"].view(np.uint64))
    _check_compact(h, osch.compact_pi(o["mask"], o["pi"], cu, B))
    pi = si.draw_inclusion_probs(N, seed=3)
    m = osch.select_poisson(cu, pi, seed=8, step=1, drop_zero_adv=adv)
    h = stage.select_compact(params, to_dev(cu), B, N, B, poisson_pi=to_dev(pi))
    assert _mask_words(h, m)
    _check_compact(h, osch.compact_pi(m, pi, cu, B))


# ---------------------------------------------------------------- prefix packing

def _pack_both(stage, P, cu, cut, shift, ids=None):
    B, N = len(cu) - 1, int(cu[-1])
    rows_cap = int((0 if P is None else int(np.sum(P))) + N)
    o = osch.prefix_pack(P, cu, cut, shift)
    h = stage.prefix_pack(None if P is None else to_dev(np.asarray(P, np.int32)), to_dev(cu),
                          to_dev(np.asarray(cut, np.int32)), B, N, rows_cap, shift,
                          None if ids is None else to_dev(ids))
    M, K = o["total"], len(o["loss_row"])
    assert (h["total"], h["max_len"]) == (M, o["max_len"])
    assert h["totals"].cpu().numpy().tolist() == [M, o["max_len"]]
    assert np.array_equal(h["cu_packed"].cpu().numpy(), o["cu_packed"])
    assert int(h["cu_loss"][-1]) == K
    assert np.array_equal(h["src_idx"].cpu().numpy()[:M], o["src_idx"])
    assert np.array_equal(h["position_ids"].cpu().numpy()[:M], o["position_ids"])
    assert np.array_equal(h["loss_row"].cpu().numpy()[:K], o["loss_row"])
    if ids is not None:
        assert np.array_equal(h["input_ids_packed"].cpu().numpy()[:M], ids[o["src_idx"]])
    return h, o


@pytest.mark.parametrize("shift", [0, 1])
def test_prefix_pack_edge_cases(stage, shift):
    T = np.array([5, 0, 9, 1, 30, 1025, 1, 0, 64])
    P = np.array([3, 2, 1, 4, 7, 1, 1, 5, 300])
    cu = np.concatenate([[0], np.cumsum(T)]).astype(np.int64)
    ids = np.random.default_rng(1).integers(0, 50000, int(T.sum() + P.sum())).astype(np.int32)
    for cut in (np.array([2, 0, 9, 0, 11, 1000, 1, 0, 1]), T.copy(), np.zeros_like(T)):
        _pack_both(stage, P, cu, cut, shift, ids)
    if shift == 0:
        _pack_both(stage, None, cu, T, 0)                           # no prompts, nothing cut: identity


def test_prefix_pack_many_rollouts_spans_scan_chunks(stage):
    rng = np.random.default_rng(2)
    B = 2500                                                        # more than two 1024-wide scan chunks
    T = rng.integers(0, 40, B)
    P = rng.integers(1, 9, B)
    cu = np.concatenate([[0], np.cumsum(T)]).astype(np.int64)
    cut = (T * rng.random(B)).astype(np.int64)
    _pack_both(stage, P, cu, cut, 1)


def test_prefix_pack_full_size_after_rpc_select(stage):
    import paper_2603_06619_amd as nat
    lay = si.batch_layout("qwen3_8b_head_rpc", 2000)
    cu, B, N = lay["cu_seqlens"], lay["B"], lay["N"]
    P = si.draw_prompt_lengths(B, seed=3)
    sel = stage.select_compact(nat.SelectParams(nat.RPC, min_cut=1, seed=77, step=1), to_dev(cu), B, N, B)
    o_sel = osel.select(cu, osel.RPC, C=1, seed=77, step=1)
    h, o = _pack_both(stage, P, cu, o_sel["cut_len"], 1)
    # the packer's kept-token offsets are the compaction's, and it drops about half of the response rows
    assert torch.equal(h["cu_loss"], sel["cu_kept"])
    assert 0.4 < (o["total"] - int(P.sum())) / N < 0.6


def test_prefix_pack_clamps_cuts_outside_the_rollout(stage):
    T = np.array([4, 6])
    cu = np.concatenate([[0], np.cumsum(T)]).astype(np.int64)
    h = stage.prefix_pack(None, to_dev(cu), to_dev(np.array([-3, 99], np.int32)), 2, 10, 10, 0)
    assert h["cu_packed"].cpu().numpy().tolist() == [0, 0, 6] and h["total"] == 6


# ---------------------------------------------------------------- through the loss

def test_schedule_selected_tokens_through_the_loss(stage):
    # select by schedule -> compact with the survival weights -> loss and gradients, against the
    # oracle's estimate (Eq. 9) for the same mask and probabilities
    rng = np.random.default_rng(6)
    lengths = [40, 1, 75, 0, 33]
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    B, N, H, V = len(lengths), int(cu[-1]), 128, 640
    case = make_loss_case(11, N, H, V, "bf16", n_seq=B)
    adv = rng.standard_normal(B).astype(np.float32)
    w = si.draw_schedule_weights(lengths, "tail_mass", seed=4)
    o = osch.select_schedule(cu, w, seed=21, step=0)
    batch = dict(cu_seqlens=cu, hidden=case["hidden"].astype(np.float64), W=case["W"].astype(np.float64),
                 ids=case["ids"], old_logp=case["old_logp"].astype(np.float64), adv=adv.astype(np.float64))
    ref = odrv.estimate(batch, o["mask"], o["pi"])
    hidden = to_dev(case["hidden"], torch.bfloat16)
    h = stage.select_compact(_params(21, 0), to_dev(cu), B, N, B, hidden=hidden, ids=to_dev(case["ids"]),
                             old_logp=to_dev(case["old_logp"]), schedule_weights=to_dev(w.view(np.int32)))
    nk = h["n_kept"]
    out = stage.loss(h["hidden_k"], to_dev(case["W"], torch.bfloat16), h["ids_k"], h["old_logp_k"], to_dev(adv),
                     h["kept_seq"], h["kept_w"], nk)
    torch.cuda.synchronize()
    assert abs(float(out["loss"]) - ref["loss"]) <= 2e-2 * abs(ref["loss"])
    kept = np.nonzero(o["mask"])[0]
    assert max_rel_err(out["dH"][:nk].float().cpu().numpy(), ref["dH"][kept]) < 2e-2
    assert max_rel_err(out["dW"].cpu().numpy(), ref["dW"]) < 2e-2
