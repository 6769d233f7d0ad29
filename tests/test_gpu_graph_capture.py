"""The library calls only enqueue kernels (and one small pinned copy) on the caller's stream, allocate
nothing and clear memory with a fill kernel, so a caller can record them into a HIP graph.  The loss call
and the selection calls are captured, replayed several times with eager work in between, and every replay
is compared bit for bit with the eager result."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from nat_testlib import DEV, make_loss_case, to_dev


def test_loss_call_replays_from_a_graph_bit_for_bit():
    import paper_2603_06619_amd as nat
    n, H, V = 700, 256, 5000
    case = make_loss_case(5, n, H, V, "bf16", noise=0.1, w_std=0.1)
    t = {k: to_dev(v, torch.bfloat16 if k in ("hidden", "W") else None) for k, v in case.items()}
    ws = torch.empty(nat.loss_workspace_bytes(n, H, V, nat.DTYPE_BF16), dtype=torch.uint8, device=DEV)
    mk = lambda: dict(loss=torch.zeros(1, device=DEV), logp=torch.zeros(n, device=DEV),
                      dH=torch.zeros((n, H), dtype=torch.bfloat16, device=DEV), dW=torch.zeros((V, H), device=DEV))
    call = lambda o: nat.nat_loss_fwd_bwd(t["hidden"], t["W"], t["ids"], t["old_logp"], t["adv"], t["kept_seq"],
                                          t["kept_w"], n, 0.2, 0.2, 1.0, o["loss"], o["logp"], o["dH"], o["dW"],
                                          False, ws)
    eager = mk()
    call(eager)
    torch.cuda.synchronize()
    ref = {k: v.clone() for k, v in eager.items()}
    out = mk()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call(out)                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call(out)
    for rep in range(4):
        for v in out.values():
            v.fill_(7.0)                            # eager work between replays; outputs must be rewritten
        ws.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k in ref:
            assert torch.equal(out[k], ref[k]), (rep, k)


def test_selection_calls_replay_from_a_graph():
    import paper_2603_06619_amd as nat
    lengths = np.array([300, 1, 70, 1030, 0, 64, 4097])
    cu = to_dev(np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64))
    B, N = len(lengths), int(lengths.sum())
    params = nat.SelectParams(nat.URS, p=0.5, seed=11, step=2)
    i32 = lambda k: torch.zeros(max(k, 1), dtype=torch.int32, device=DEV)
    bufs = dict(cut=i32(B), mask=i32(nat.mask_words(N)), idx=i32(N), seq=i32(N), w=torch.zeros(N, device=DEV),
                cuk=i32(B + 1), nk=i32(1))
    h_nk = torch.zeros(1, dtype=torch.int32).pin_memory()
    ws = torch.empty(nat.compact_workspace_bytes(N), dtype=torch.uint8, device=DEV)

    def call():
        nat.nat_select(params, cu, B, N, bufs["cut"], bufs["mask"])
        nat.nat_compact(params, B, bufs["mask"], cu, B, N, bufs["idx"], bufs["seq"], bufs["w"], bufs["cuk"], bufs["nk"],
                        h_nk, ws)
    call()
    torch.cuda.synchronize()
    ref = {k: v.clone() for k, v in bufs.items()}
    nk_ref = int(h_nk[0])
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call()
    for rep in range(3):
        for v in bufs.values():
            v.fill_(0)
        h_nk.fill_(-1)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert int(h_nk[0]) == nk_ref
        for k in ("cut", "mask", "cuk", "nk"):
            assert torch.equal(bufs[k], ref[k]), (rep, k)
        for k in ("idx", "seq", "w"):
            assert torch.equal(bufs[k][:nk_ref], ref[k][:nk_ref]), (rep, k)
