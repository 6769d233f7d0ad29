"""Shared helpers of the GPU parity tests: run the oracle and the HIP path on the
same seeded inputs and compare."""
import numpy as np
import torch

import synth_inputs as si
from oracle import grpo as ogrpo
from oracle import select as osel

DEV = "cuda:0"


def max_rel_err(got, ref):
    """||got - ref||_inf / ||ref||_inf  (the tolerance metric of the parity bar)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.abs(ref).max()
    return float(np.abs(got - ref).max() / den) if den > 0 else float(np.abs(got).max())


def rel_frobenius(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / den) if den > 0 else float(np.linalg.norm(got))


def dh_residual_error(dH_got, ref, W, ids, out_ulp):
    """(error of dH with the one-hot term c_k W[y_k] removed on both sides, over the largest residual
    entry of the oracle; that largest entry).  See contraction_errors."""
    ids = np.asarray(ids, dtype=np.int64)
    W_rows = np.asarray(W[ids], dtype=np.float64)
    res_ref = ref["dH"] - ref["c"][:, None] * W_rows
    diff = np.abs(np.asarray(dH_got, dtype=np.float64) - ref["dH"]) - out_ulp * np.abs(ref["dH"])
    den = np.abs(res_ref).max()
    err = float(np.maximum(diff, 0.0).max())
    return (err / den if den > 0 else err), den


def contraction_errors(dH_got, dW_got, ref, hidden, W, ids, out_ulp):
    """Errors of the parts of dH and dW that only the two backward contractions produce.

    dz_k = c_k (onehot(y_k) - softmax_k) splits each gradient into the one-hot term (c_k W[y_k] in
    dH_k, c_k h_k added to row y_k of dW) and the soft-max term (-c_k sum_v p_kv W_v, resp.
    -sum_k c_k p_kv h_k).  With a near-uniform soft-max the one-hot term dominates the tensors'
    maxima, so a max-norm over the whole tensor says little about the contractions.  Here:
      dW_off  rows of dW no token targets (soft-max term alone): ||got - ref||_inf over those rows,
              divided by the largest off-target entry of the oracle;
      dH_res  dH with the one-hot term c_k W[y_k] (oracle's c_k, fp64) taken off both sides,
              divided by the largest entry of the oracle's residual.  dH is stored in the input
              element type, so each entry also carries the rounding of the FULL value:
              out_ulp * |dH_ref| (the caller's figure for that rounding) is allowed on top, entry by entry;
              the returned figure is max over entries of (|diff| - out_ulp |dH_ref|)+ / max|residual|.
    Also relative Frobenius errors of the whole tensors (reported, not asserted)."""
    ids = np.asarray(ids, dtype=np.int64)
    W64 = np.asarray(W, dtype=np.float64)
    dH_got = np.asarray(dH_got, dtype=np.float64)
    dW_got = np.asarray(dW_got, dtype=np.float64)
    dH_res, den = dh_residual_error(dH_got, ref, W64, ids, out_ulp)
    off = np.ones(W64.shape[0], dtype=bool)
    off[ids] = False
    if off.any():
        den_off = np.abs(ref["dW"][off]).max()
        dW_off = float(np.abs(dW_got[off] - ref["dW"][off]).max() / den_off) if den_off > 0 else 0.0
        off_share = float(den_off / np.abs(ref["dW"]).max())
    else:
        dW_off, off_share = 0.0, 1.0
    return dict(dH_res=dH_res, dW_off=dW_off, dW_off_share=off_share,
                dH_res_share=float(den / np.abs(ref["dH"]).max()) if np.abs(ref["dH"]).max() > 0 else 0.0,
                dH_fro=rel_frobenius(dH_got, ref["dH"]), dW_fro=rel_frobenius(dW_got, ref["dW"]))


def to_dev(x, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(x))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV)


def oracle_select_compact(cu, scheme, n_rollouts=None, p=1.0, C=1, beta=1.0, seed=0, step=0, base=0, spr=None,
                          drop=None):
    B = len(cu) - 1
    d = osel.select(cu, scheme, p=p, C=C, beta=beta, seed=seed, step=step, rollout_id_base=base,
                    scheme_per_rollout=spr, drop_zero_adv=drop)
    c = osel.compact(d["mask"], cu, B if n_rollouts is None else n_rollouts, scheme, p=p, C=C,
                     scheme_per_rollout=spr)
    c.update(d)
    return c


def hip_select_compact(stage, cu, scheme, n_rollouts=None, p=1.0, C=1, beta=1.0, seed=0, step=0, base=0, spr=None,
                       hidden=None, ids=None, old_logp=None, drop=None):
    import paper_2603_06619_amd as nat
    B = len(cu) - 1
    N = int(cu[-1])
    params = nat.SelectParams(scheme, p=p, min_cut=C, trunc_frac=beta, seed=seed, step=step, rollout_id_base=base,
                              scheme_per_rollout=to_dev(np.asarray(spr, dtype=np.int32)) if spr is not None else None,
                              drop_zero_adv=to_dev(np.asarray(drop, dtype=np.float32)) if drop is not None else None)
    out = stage.select_compact(params, to_dev(np.asarray(cu, dtype=np.int64)), B, N, n_rollouts, hidden, ids, old_logp)
    return out


def assert_select_compact_equal(h, o, N):
    nk = o["n_kept"]
    assert h["n_kept"] == nk
    assert int(h["n_kept_dev"].item()) == nk
    assert np.array_equal(h["cut_len"].cpu().numpy(), o["cut_len"])
    words = h["mask_bits"].cpu().numpy().view(np.uint32)
    assert np.array_equal(words[:len(osel.pack_mask_bits(o["mask"]))], osel.pack_mask_bits(o["mask"]))
    assert np.array_equal(h["kept_idx"].cpu().numpy()[:nk], o["kept_idx"])
    assert np.array_equal(h["kept_seq"].cpu().numpy()[:nk], o["kept_seq"])
    assert np.array_equal(h["cu_kept"].cpu().numpy(), o["cu_kept"])
    # weights: one fp64 division rounded to fp32 on both sides -> identical bits
    assert np.array_equal(h["kept_w"].cpu().numpy()[:nk].view(np.uint32), o["kept_w"].view(np.uint32))


def oracle_loss(hidden, W, ids, old_logp, adv, kept_seq, kept_w, eps_lo=0.2, eps_hi=0.2, grad_scale=1.0, **kl):
    return ogrpo.loss_and_grads(hidden, W, ids, old_logp, np.asarray(adv, np.float64)[kept_seq],
                                np.asarray(kept_w, np.float64), eps_lo, eps_hi, grad_scale, **kl)


def make_loss_case(seed, n_tok, H, V, dtype, n_seq=4, noise=0.05, w_std=0.02):
    """Kept-token inputs for nat_loss_fwd_bwd drawn directly (no selection): numpy float32 arrays
    (bf16-representable when dtype is bf16)."""
    rng = np.random.default_rng(seed)
    hidden = rng.standard_normal((n_tok, H), dtype=np.float32)
    W = rng.standard_normal((V, H), dtype=np.float32) * np.float32(w_std)
    if dtype == "bf16":
        hidden, _ = si.round_to_bf16(hidden)
        W, _ = si.round_to_bf16(W)
    ids = rng.integers(0, V, n_tok).astype(np.int32)
    kept_seq = np.sort(rng.integers(0, n_seq, n_tok)).astype(np.int32)
    adv = rng.standard_normal(n_seq).astype(np.float32)
    adv[0] = 0.0                                   # a zero-advantage rollout
    kept_w = (rng.random(n_tok) * 1e-3 + 1e-4).astype(np.float32)
    logp = ogrpo.token_logp(hidden, W, ids)        # current log-probs from the oracle (fp64)
    old_logp = (logp + rng.standard_normal(n_tok) * noise).astype(np.float32)
    return dict(hidden=hidden, W=W, ids=ids, kept_seq=kept_seq, adv=adv, kept_w=kept_w, old_logp=old_logp)


def hip_loss(stage, case, dtype, **kw):
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    n = len(case["ids"])
    out = stage.loss(to_dev(case["hidden"], tdt), to_dev(case["W"], tdt), to_dev(case["ids"]),
                     to_dev(case["old_logp"]), to_dev(case["adv"]), to_dev(case["kept_seq"]), to_dev(case["kept_w"]),
                     n, **kw)
    torch.cuda.synchronize()
    return out


def behaviour_logp_from_forward(stage, batch, n_spot=24, seed=0):
    """Behaviour-policy log-probs of a full-size device batch: the current policy's log-prob of every
    token (the forward pass alone, nat_logp_fwd, over all N tokens) plus the batch's N(0, 0.05) noise.
    A random subsample of the forward log-probs is checked against the oracle (fp64, token by token)."""
    N = batch["N"]
    lp = stage.logp(batch["hidden"], batch["W"], batch["ids"], N)["logp"][:N]
    torch.cuda.synchronize()
    spot = np.unique(np.concatenate([[0, N - 1], np.random.default_rng(seed).integers(0, N, n_spot)]))
    sidx = torch.from_numpy(spot).to(batch["hidden"].device)
    ref = ogrpo.token_logp(batch["hidden"][sidx].float().cpu().numpy(), batch["W"].float().cpu().numpy(),
                           batch["ids"][sidx].cpu().numpy())
    tol = 1e-4 if batch["dtype"] == "bf16" else 1e-5 * float(np.abs(ref).max())
    err = float(np.abs(lp[sidx].cpu().numpy().astype(np.float64) - ref).max())
    assert err <= tol, ("forward log-probs against the oracle", err)
    return lp + batch["logp_noise"]
