"""nat_compact_static (the entry point that allocates nothing: its scratch is part of the library's
device image) against nat_compact, through the C ABI, bit for bit: two calls in a row on the same
GPU, the second on a smaller batch, so that stale contents of the shared scratch would show."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import synth_inputs as si
from nat_testlib import DEV, to_dev


def _run(nat, entry, params, cu, B, N, hidden, ids, old):
    i32 = lambda n: torch.full((max(int(n), 1),), -3, dtype=torch.int32, device=DEV)
    o = dict(idx=i32(N), seq=i32(N), w=torch.full((max(N, 1),), -3.0, dtype=torch.float32, device=DEV), cuk=i32(B + 1),
             nk=i32(1), hk=torch.full((max(N, 1), hidden.shape[1]), -3.0, dtype=hidden.dtype, device=DEV),
             idk=i32(N), olk=torch.full((max(N, 1),), -3.0, dtype=torch.float32, device=DEV))
    h_nk = torch.full((1,), -1, dtype=torch.int32).pin_memory()
    cut, mask = i32(B), i32(nat.mask_words(N))
    nat.nat_select(params, cu, B, N, cut, mask)
    if entry == "static":
        nat.nat_compact_static(params, B, mask, cu, B, N, o["idx"], o["seq"], o["w"], o["cuk"], o["nk"], h_nk,
                               hidden, o["hk"], ids, o["idk"], old, o["olk"])
    else:
        ws = torch.empty(nat.compact_workspace_bytes(N), dtype=torch.uint8, device=DEV)
        nat.nat_compact(params, B, mask, cu, B, N, o["idx"], o["seq"], o["w"], o["cuk"], o["nk"], h_nk, ws,
                        hidden, o["hk"], ids, o["idk"], old, o["olk"])
    torch.cuda.synchronize()
    o["h_nk"] = int(h_nk[0])
    return o


def test_static_scratch_entry_point_matches_nat_compact_on_two_calls_in_a_row():
    import paper_2603_06619_amd as nat
    rng = np.random.default_rng(0)
    # first a batch of several hundred mask tiles, then a much smaller one (fewer tiles than before)
    cases = [(("uniform", 2000, 9000), 64, nat.URS, dict(p=0.5)), (("uniform", 1, 700), 5, nat.RPC, dict(min_cut=3))]
    for lengths, B, scheme, kw in cases:
        lay = si.batch_layout("qwen3_0p6b_head", 7, P=1, G=B, lengths=lengths)
        cu, N = to_dev(lay["cu_seqlens"]), lay["N"]
        hidden = to_dev(rng.standard_normal((N, 64)).astype(np.float32), torch.bfloat16)
        ids = to_dev(rng.integers(0, 50000, N).astype(np.int32))
        old = to_dev(rng.standard_normal(N).astype(np.float32))
        params = nat.SelectParams(scheme, seed=9, step=3, **kw)
        got = _run(nat, "static", params, cu, B, N, hidden, ids, old)
        ref = _run(nat, "workspace", params, cu, B, N, hidden, ids, old)
        assert got["h_nk"] == ref["h_nk"] > 0 and int(got["nk"].item()) == ref["h_nk"]
        for k in ("idx", "seq", "w", "cuk", "hk", "idk", "olk"):
            assert torch.equal(got[k], ref[k]), (k, lengths)


def test_static_scratch_entry_point_rejects_batches_beyond_its_scratch():
    import ctypes
    import paper_2603_06619_amd as nat
    params = nat.SelectParams(nat.URS, p=0.5)
    with pytest.raises(nat.NatError) as e:
        nat.nat_compact_static(params, 4, None, None, 4, (1 << 28) + 1, None, None, None, None, None, None)
    assert e.value.status == 2
