"""GPU tests of what the library does with values it can only see on the device: a host-passed
token count larger than cu_seqlens[B], a kept-token capacity smaller than the number kept, token
ids outside the vocabulary, and the diagnostic counters of nat_loss_fwd_bwd_kl / nat_logp_fwd.
Every case here is one the kernels bound themselves: nothing below is out of range on the device."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import synth_inputs as si
from oracle import grpo as ogrpo
from oracle import select as osel
from nat_testlib import (DEV, contraction_errors, hip_loss, make_loss_case, max_rel_err, oracle_loss,
                         oracle_select_compact, to_dev)


@pytest.fixture(scope="module")
def stage():
    from paper_2603_06619_amd.stage import LossStage
    return LossStage(DEV)


def _select_buffers(nat, B, N_alloc):
    i32 = lambda n: torch.full((max(int(n), 1),), -7, dtype=torch.int32, device=DEV)
    return dict(cut=i32(B), mask=i32(nat.mask_words(N_alloc)), idx=i32(N_alloc), seq=i32(N_alloc),
                w=torch.full((max(N_alloc, 1),), -7.0, dtype=torch.float32, device=DEV), cuk=i32(B + 1), nk=i32(1),
                ws=torch.empty(nat.compact_workspace_bytes(N_alloc), dtype=torch.uint8, device=DEV))


@pytest.mark.parametrize("scheme,kw", [(osel.URS, dict(p=0.5)), (osel.RPC, dict(C=3)), (osel.FULL, {})])
def test_host_token_count_larger_than_the_offsets_say(scheme, kw):
    # the caller sizes its arrays for N_alloc tokens but the offsets end at N < N_alloc: positions in
    # [N, N_alloc) belong to no rollout and are never kept; everything else is as for the exact N
    import paper_2603_06619_amd as nat
    lengths = [300, 0, 1, 777, 64, 1030]
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    B, N = len(lengths), int(cu[-1])
    N_alloc = N + 5000                                    # several mask tiles past the end
    o = oracle_select_compact(cu, scheme, p=kw.get("p", 1.0), C=kw.get("C", 1), seed=11, step=2)
    params = nat.SelectParams(scheme, p=kw.get("p", 1.0), min_cut=kw.get("C", 1), seed=11, step=2)
    b = _select_buffers(nat, B, N_alloc)
    d_cu = to_dev(cu)
    nat.nat_select(params, d_cu, B, N_alloc, b["cut"], b["mask"])
    nat.nat_compact(params, B, b["mask"], d_cu, B, N_alloc, b["idx"], b["seq"], b["w"], b["cuk"], b["nk"], None, b["ws"])
    torch.cuda.synchronize()
    nk = o["n_kept"]
    assert int(b["nk"].item()) == nk
    bits = np.unpackbits(b["mask"].cpu().numpy().view(np.uint8), bitorder="little")
    assert np.array_equal(bits[:N].astype(bool), o["mask"]) and not bits[N:].any()
    assert np.array_equal(b["idx"].cpu().numpy()[:nk], o["kept_idx"])
    assert np.array_equal(b["seq"].cpu().numpy()[:nk], o["kept_seq"])
    assert np.array_equal(b["w"].cpu().numpy()[:nk].view(np.uint32), o["kept_w"].view(np.uint32))
    assert np.array_equal(b["cuk"].cpu().numpy(), o["cu_kept"])
    assert (b["idx"][nk:] == -7).all()                   # nothing written past the kept tokens


def test_schedule_and_poisson_with_a_larger_host_token_count():
    import paper_2603_06619_amd as nat
    from oracle import schedule as osch
    lengths = [500, 3, 0, 1200]
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    B, N = len(lengths), int(cu[-1])
    N_alloc = N + 3000
    w = si.draw_schedule_weights(lengths, "random", seed=4)
    o = osch.select_schedule(cu, w, seed=3, step=1)
    params = nat.SelectParams(nat.FULL, seed=3, step=1)
    b = _select_buffers(nat, B, N_alloc)
    pi = torch.full((N_alloc,), -1.0, dtype=torch.float64, device=DEV)
    w_dev = torch.zeros(N_alloc, dtype=torch.int32, device=DEV)
    w_dev[:N] = to_dev(w.view(np.int32))
    nat.nat_select_schedule(params, w_dev, to_dev(cu), B, N_alloc, b["cut"], b["mask"], pi)
    torch.cuda.synchronize()
    assert np.array_equal(b["cut"].cpu().numpy(), o["cut_len"])
    bits = np.unpackbits(b["mask"].cpu().numpy().view(np.uint8), bitorder="little")
    assert np.array_equal(bits[:N].astype(bool), o["mask"]) and not bits[N:].any()
    assert np.array_equal(pi.cpu().numpy()[:N].view(np.uint64), o["pi"].view(np.uint64))
    assert (pi[N:] == -1.0).all()
    p_tok = np.ones(N_alloc)
    p_tok[:N] = si.draw_inclusion_probs(N, seed=5)
    m = osch.select_poisson(cu, p_tok[:N], seed=3, step=1)
    nat.nat_select_poisson(params, to_dev(p_tok), to_dev(cu), B, N_alloc, b["mask"])
    torch.cuda.synchronize()
    bits = np.unpackbits(b["mask"].cpu().numpy().view(np.uint8), bitorder="little")
    assert np.array_equal(bits[:N].astype(bool), m) and not bits[N:].any()     # p = 1 beyond the end: still not kept


def test_kept_token_capacity_bounds_every_output():
    # capacity below the number of kept tokens: the first `cap` entries are the usual ones, nothing
    # is written beyond them, and n_kept still reports the true count
    import paper_2603_06619_amd as nat
    lay = si.batch_layout("qwen3_0p6b_head", 5, P=2, G=4, lengths=("uniform", 700, 3000))
    cu, B, N = lay["cu_seqlens"], lay["B"], lay["N"]
    o = oracle_select_compact(cu, osel.URS, p=0.5, seed=21)
    nk = o["n_kept"]
    cap = nk - 1234
    H = 64
    rng = np.random.default_rng(0)
    hidden = rng.standard_normal((N, H)).astype(np.float32)
    ids = rng.integers(0, 1000, N).astype(np.int32)
    old = rng.standard_normal(N).astype(np.float32)
    params = nat.SelectParams(nat.URS, p=0.5, seed=21)
    b = _select_buffers(nat, B, N)
    hk = torch.full((N, H), -7.0, dtype=torch.float32, device=DEV)
    idk = torch.full((N,), -7, dtype=torch.int32, device=DEV)
    olk = torch.full((N,), -7.0, dtype=torch.float32, device=DEV)
    d_cu = to_dev(cu)
    nat.nat_select(params, d_cu, B, N, b["cut"], b["mask"])
    nat.nat_compact(params, B, b["mask"], d_cu, B, N, b["idx"], b["seq"], b["w"], b["cuk"], b["nk"], None, b["ws"],
                    to_dev(hidden), hk, to_dev(ids), idk, to_dev(old), olk, kept_cap=cap)
    torch.cuda.synchronize()
    assert int(b["nk"].item()) == nk > cap
    assert np.array_equal(b["cuk"].cpu().numpy(), o["cu_kept"])
    k = o["kept_idx"][:cap]
    assert np.array_equal(b["idx"].cpu().numpy()[:cap], k)
    assert np.array_equal(b["seq"].cpu().numpy()[:cap], o["kept_seq"][:cap])
    assert np.array_equal(b["w"].cpu().numpy()[:cap].view(np.uint32), o["kept_w"][:cap].view(np.uint32))
    assert np.array_equal(hk.cpu().numpy()[:cap], hidden[k]) and np.array_equal(idk.cpu().numpy()[:cap], ids[k])
    assert np.array_equal(olk.cpu().numpy()[:cap], old[k])
    for t in (b["idx"], b["seq"], idk):
        assert (t[cap:] == -7).all()
    assert (b["w"][cap:] == -7.0).all() and (hk[cap:] == -7.0).all() and (olk[cap:] == -7.0).all()
    # capacity zero: only the counts
    b0 = _select_buffers(nat, B, N)
    nat.nat_compact(params, B, b["mask"], d_cu, B, N, None, None, None, b0["cuk"], b0["nk"], None, b0["ws"], kept_cap=0)
    torch.cuda.synchronize()
    assert int(b0["nk"].item()) == nk and np.array_equal(b0["cuk"].cpu().numpy(), o["cu_kept"])


@pytest.mark.parametrize("dtype,H,V,n_tok,tol", [("bf16", 128, 3000, 700, 2e-2), ("f32", 64, 512, 90, 1e-5)])
def test_token_ids_outside_the_vocabulary_are_left_out_and_counted(stage, dtype, H, V, n_tok, tol):
    import paper_2603_06619_amd as nat
    case = make_loss_case(61, n_tok, H, V, dtype, noise=0.1, w_std=0.1)
    bad = np.array([0, 5, 255, 256, n_tok - 1, n_tok // 2])
    bad = bad[bad < n_tok]
    good = np.setdiff1d(np.arange(n_tok), bad)
    ref = oracle_loss(**{k: (v[good] if k in ("hidden", "ids", "kept_seq", "kept_w", "old_logp") else v)
                         for k, v in case.items()})
    broken = dict(case)
    broken["ids"] = case["ids"].copy()
    broken["ids"][bad] = [V, -1, V + 300, 2 ** 31 - 1, -2 ** 31, V][:len(bad)]
    ws = nat.loss_workspace_min_bytes(n_tok, H, V, nat.DTYPE_BF16 if dtype == "bf16" else nat.DTYPE_F32)
    for ws_bytes in (None, ws):                            # one chunk, and 256-token (resp. 1-token) chunks
        out = hip_loss(stage, broken, dtype, want_diag=True, want_entropy=True, ws_bytes=ws_bytes)
        diag = out["diag"].cpu().numpy()
        assert diag[nat.DIAG_BAD_ID] == len(bad) and diag[nat.DIAG_SHIFT_RANGE] == 0
        logp = out["logp"].cpu().numpy()[:n_tok]
        assert np.isnan(logp[bad]).all() and np.isfinite(logp[good]).all()
        assert np.abs(logp[good] - ref["logp"]).max() <= (1e-4 if dtype == "bf16" else 1e-5 * np.abs(ref["logp"]).max())
        dH = out["dH"].float().cpu().numpy()[:n_tok]
        assert not dH[bad].any()                            # rows of the left-out tokens are exactly zero
        assert max_rel_err(dH[good], ref["dH"]) <= tol
        assert max_rel_err(out["dW"].cpu().numpy(), ref["dW"]) <= tol
        assert abs(out["loss"].item() - ref["loss"]) <= max(tol * 5e-3, 1e-5) * abs(ref["loss"])
        # the entropy does not depend on the target: defined for every row
        ent_all = ogrpo.forward_logp(case["hidden"], case["W"], case["ids"])["entropy"]
        assert max_rel_err(out["entropy"].cpu().numpy()[:n_tok], ent_all) <= 1e-4
    # forward pass alone: same rule
    lp = stage.logp(to_dev(broken["hidden"], torch.bfloat16 if dtype == "bf16" else torch.float32),
                    to_dev(broken["W"], torch.bfloat16 if dtype == "bf16" else torch.float32),
                    to_dev(broken["ids"]), n_tok, want_diag=True)
    torch.cuda.synchronize()
    d2 = lp["diag"].cpu().numpy()
    assert d2[nat.DIAG_BAD_ID] == len(bad) and d2[nat.DIAG_CLIPPED] == 0 and d2[nat.DIAG_NONZERO_ADV] == 0
    got = lp["logp"].cpu().numpy()[:n_tok]
    assert np.isnan(got[bad]).all() and np.abs(got[good] - ref["logp"]).max() <= 1e-4


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_clip_counters_match_the_oracle(stage, dtype):
    import paper_2603_06619_amd as nat
    H, V, n_tok = (128, 2000, 900) if dtype == "bf16" else (64, 512, 200)
    case = make_loss_case(71, n_tok, H, V, dtype, noise=0.25, w_std=0.1)      # a good share of ratios beyond 1 +- 0.2
    ref = oracle_loss(**case)
    A = case["adv"].astype(np.float64)[case["kept_seq"]]
    r = ref["r"]
    clipped_ref = ((A > 0) & (r > 1.2)) | ((A < 0) & (r < 0.8))
    near = np.minimum(np.abs(r - 1.2), np.abs(r - 0.8)) < 1e-5           # fp32 ratio may fall on the other side
    out = hip_loss(stage, case, dtype, want_diag=True)
    diag = out["diag"].cpu().numpy()
    assert diag[nat.DIAG_NONZERO_ADV] == int((A != 0).sum()) and (A == 0).any()
    assert abs(int(diag[nat.DIAG_CLIPPED]) - int(clipped_ref.sum())) <= int(near.sum())
    assert clipped_ref.sum() > 20 and diag[nat.DIAG_BAD_ID] == 0 and diag[nat.DIAG_SHIFT_RANGE] == 0
    # the counters are cleared by every call, also one without tokens
    W = to_dev(case["W"], torch.bfloat16 if dtype == "bf16" else torch.float32)
    dW = torch.zeros((V, H), dtype=torch.float32, device=DEV)
    loss = torch.zeros(1, dtype=torch.float32, device=DEV)
    stale = torch.full((nat.DIAG_WORDS,), 9, dtype=torch.int32, device=DEV)
    nat.nat_loss_fwd_bwd_kl(None, W, None, None, None, None, None, 0, 0.2, 0.2, 1.0, None, 0.0, 0, loss, None, None,
                            None, None, dW, False, None, stale)
    torch.cuda.synchronize()
    assert not stale.any()


def test_shift_range_counter_flags_tokens_beyond_the_bound(stage):
    # bf16 path: the exponent shift is the target logit, valid while log(p_max / p_target) < 70.  Build rows
    # whose target sits far below the mode: logits spread over about +-60, so some tokens exceed the bound.
    import paper_2603_06619_amd as nat
    n_tok, H, V = 600, 128, 2000
    case = make_loss_case(81, n_tok, H, V, "bf16", noise=0.1, w_std=1.5)
    Z = case["hidden"].astype(np.float64) @ case["W"].astype(np.float64).T
    ids = case["ids"].copy()
    ids[::3] = Z[::3].argmin(axis=1)                       # the least likely token: the largest gap
    case["ids"] = ids.astype(np.int32)
    gap = Z.max(axis=1) - Z[np.arange(n_tok), ids]
    beyond = gap >= 70.0 + np.log(128.0)                   # certainly flagged: one numerator alone reaches e^70
    within = gap < 70.0 - 1e-3                             # certainly not: even 128 of them stay below... see below
    assert beyond.sum() > 20 and within.sum() > 100
    out = stage.logp(to_dev(case["hidden"], torch.bfloat16), to_dev(case["W"], torch.bfloat16), to_dev(case["ids"]),
                     n_tok, want_diag=True)
    torch.cuda.synchronize()
    flagged = int(out["diag"].cpu().numpy()[nat.DIAG_SHIFT_RANGE])
    # a granule's sum reaches e^70 iff sum_v exp(z_v - z_y) over its 128 rows does: computed here in fp64
    v_blocks = [slice(a, min(a + 128, V)) for a in range(0, V, 128)]
    expect = np.zeros(n_tok, dtype=bool)
    margin = np.zeros(n_tok, dtype=bool)
    for sl in v_blocks:
        s = np.exp(np.minimum(Z[:, sl] - Z[np.arange(n_tok), ids][:, None], 70.0)).sum(axis=1)
        expect |= s >= np.exp(70.0)
        margin |= np.abs(np.log(s) - 70.0) < 1e-3          # too close to call in fp32
    assert expect[beyond].all() and expect.sum() > 20
    assert abs(flagged - int(expect.sum())) <= int(margin.sum())
    # tokens inside the bound keep their accuracy next to flagged ones
    ref = ogrpo.forward_logp(case["hidden"], case["W"], case["ids"])
    ok = gap < 60.0
    assert np.abs(out["logp"].cpu().numpy()[:n_tok][ok] - ref["logp"][ok]).max() <= 2e-3
