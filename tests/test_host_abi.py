"""Host-only checks of the C-ABI library: it loads, exports every symbol that
include/nat.h declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2603_06619_amd as nat
    if not os.path.exists(nat.library_path()):
        from paper_2603_06619_amd import build
        build.build()
    return nat.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "nat.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(nat_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"nat_advantage", "nat_select", "nat_compact", "nat_loss_fwd_bwd", "nat_status_string",
            "nat_loss_workspace_bytes", "nat_compact_workspace_bytes"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings(lib):
    assert lib.nat_status_string(0) == b"NAT_OK"
    assert lib.nat_status_string(3) == b"NAT_WORKSPACE_TOO_SMALL"
    assert lib.nat_status_string(77) == b"NAT_UNKNOWN_STATUS"


def test_size_queries(lib):
    assert lib.nat_mask_words(0) == 0 and lib.nat_mask_words(1) == 2 and lib.nat_mask_words(64) == 2
    assert lib.nat_mask_words(65) == 4
    assert lib.nat_compact_workspace_bytes(1 << 20) >= (2 * 256 + 1) * 4
    big = lib.nat_loss_workspace_bytes(100000, 4096, 151936, 1)
    small = lib.nat_loss_workspace_min_bytes(100000, 4096, 151936, 1)
    assert 0 < small < big < 32 * 2 ** 30
    # the recommended workspace is bounded in N_k: chunks of 16384 tokens at H = 4096 (E = 16384 x Vp x 2 bytes
    # of about 8 GB), of 32768 tokens where 16384 would leave the dH launch with a partly filled last round
    GB = 1e9
    at_8b = lib.nat_loss_workspace_bytes(145000, 4096, 151936, 1)
    assert 7.9 * GB < at_8b < 8.1 * GB
    assert lib.nat_loss_workspace_bytes(16384, 4096, 151936, 1) <= at_8b
    assert lib.nat_loss_workspace_bytes(300000, 4096, 151936, 1) - at_8b < 1e6     # only the per-token terms grow
    assert lib.nat_loss_workspace_bytes(8000, 4096, 151936, 1) < 0.7 * at_8b        # fewer tokens than a chunk
    assert 12.9 * GB < lib.nat_loss_workspace_bytes(145000, 3584, 152064, 1) < 13.1 * GB
    assert lib.nat_logp_workspace_bytes(300000, 4096, 151936, 1) == lib.nat_logp_workspace_bytes(145000, 4096, 151936, 1)
    assert lib.nat_logp_workspace_bytes(145000, 4096, 151936, 1) < 2.0 * GB
    assert lib.nat_loss_workspace_bytes(10, 100, 512, 1) == 0          # bf16 needs H % 64 == 0
    assert lib.nat_loss_workspace_bytes(10, 64, 512, 0) > 0
    assert lib.nat_loss_workspace_bytes(10, 64, 512, 9) == 0


def _params(nat, **kw):
    from paper_2603_06619_amd.binding import _CSelectParams
    d = dict(scheme=1, min_cut=1, p=0.5, trunc_frac=0.5, seed=1, step=0, rollout_id_base=0, d_scheme_per_rollout=None)
    d.update(kw)
    return _CSelectParams(**d)


def test_select_argument_errors(lib):
    import paper_2603_06619_amd as nat
    fake = ctypes.c_void_p(256)           # never dereferenced: all of these fail validation first
    ok = _params(nat)
    assert lib.nat_select(None, fake, 4, 10, fake, fake, None) == 1
    assert lib.nat_select(ctypes.byref(ok), None, 4, 10, fake, fake, None) == 1
    assert lib.nat_select(ctypes.byref(ok), fake, 0, 10, fake, fake, None) == 1
    assert lib.nat_select(ctypes.byref(ok), fake, 4, -1, fake, fake, None) == 1
    assert lib.nat_select(ctypes.byref(ok), fake, 4, 1 << 31, fake, fake, None) == 1
    for bad in (dict(p=0.0), dict(p=1.5), dict(min_cut=0), dict(trunc_frac=0.0), dict(trunc_frac=2.0),
                dict(scheme=4), dict(scheme=-1), dict(p=float("nan"))):
        assert lib.nat_select(ctypes.byref(_params(nat, **bad)), fake, 4, 10, fake, fake, None) == 1, bad


def test_compact_argument_errors(lib):
    import paper_2603_06619_amd as nat
    fake = ctypes.c_void_p(256)
    ok = ctypes.byref(_params(nat))
    args = lambda **kw: [kw.get("params", ok), kw.get("nroll", 4), fake, fake, kw.get("B", 4), kw.get("N", 100),
                         kw.get("cap", 100), kw.get("idx", fake), fake, fake, fake, fake, None,
                         kw.get("hidden", None), kw.get("hidden_k", None), kw.get("H", 0), kw.get("dtype", 0),
                         None, None, None, None, kw.get("ws", fake), kw.get("ws_bytes", 1 << 20), None]
    assert lib.nat_compact(*args(nroll=0)) == 1
    assert lib.nat_compact(*args(B=0)) == 1
    assert lib.nat_compact(*args(hidden=fake)) == 1                       # gather pair incomplete
    assert lib.nat_compact(*args(hidden=fake, hidden_k=fake, H=3, dtype=1)) == 2   # row not 16-byte multiple
    assert lib.nat_compact(*args(hidden=fake, hidden_k=fake, H=64, dtype=5)) == 4
    assert lib.nat_compact(*args(hidden=ctypes.c_void_p(260), hidden_k=fake, H=64, dtype=1)) == 1   # misaligned rows
    assert lib.nat_compact(*args(ws_bytes=8)) == 3
    assert lib.nat_compact(*args(ws=None)) == 3
    sargs = lambda **kw: args(**kw)[:-3] + [None]                         # the variant without a workspace
    assert lib.nat_compact_static(*sargs(N=(1 << 28) + 1)) == 2           # beyond its resident scratch
    assert lib.nat_compact_static(*sargs(params=None)) == 1
    assert lib.nat_compact(*args(cap=-1)) == 1                            # negative capacity of the kept-token outputs
    assert lib.nat_compact(*args(idx=None)) == 1                          # outputs required when the capacity is positive


def test_schedule_poisson_and_pack_argument_errors(lib):
    import paper_2603_06619_amd as nat
    fake = ctypes.c_void_p(256)
    ok = ctypes.byref(_params(nat))
    assert lib.nat_select_schedule(None, fake, fake, 4, 10, fake, fake, fake, None) == 1
    assert lib.nat_select_schedule(ok, None, fake, 4, 10, fake, fake, fake, None) == 1
    assert lib.nat_select_schedule(ok, fake, None, 4, 10, fake, fake, fake, None) == 1
    assert lib.nat_select_schedule(ok, fake, fake, 0, 10, fake, fake, fake, None) == 1
    assert lib.nat_select_schedule(ok, fake, fake, 4, 1 << 31, fake, fake, fake, None) == 1
    assert lib.nat_select_schedule(ok, fake, fake, 4, 10, None, fake, fake, None) == 1
    assert lib.nat_select_schedule(ok, fake, fake, 4, 10, fake, fake, None, None) == 1
    assert lib.nat_select_poisson(ok, None, fake, 4, 10, fake, None) == 1
    assert lib.nat_select_poisson(ok, fake, fake, 4, -1, fake, None) == 1
    assert lib.nat_select_poisson(ok, fake, fake, 4, 10, None, None) == 1
    cargs = lambda **kw: [kw.get("nroll", 4), fake, kw.get("pi", fake), fake, kw.get("B", 4), 100, kw.get("cap", 100),
                          fake, fake, fake, fake, fake, None, None, None, 0, 0, None, None, None, None,
                          fake, kw.get("ws_bytes", 1 << 20), None]
    assert lib.nat_compact_pi(*cargs(pi=None)) == 1
    assert lib.nat_compact_pi(*cargs(nroll=0)) == 1
    assert lib.nat_compact_pi(*cargs(ws_bytes=8)) == 3
    assert lib.nat_compact_pi(*cargs(cap=-5)) == 1
    pargs = lambda **kw: [kw.get("P", fake), kw.get("cu", fake), fake, kw.get("B", 4), kw.get("shift", 1),
                          kw.get("rows", 100), kw.get("kept", 50), fake, fake, kw.get("src", fake), fake, fake,
                          kw.get("tot", fake), None, kw.get("ids", None), None, None]
    assert lib.nat_prefix_pack(*pargs(cu=None)) == 1
    assert lib.nat_prefix_pack(*pargs(B=0)) == 1
    assert lib.nat_prefix_pack(*pargs(shift=2)) == 1
    assert lib.nat_prefix_pack(*pargs(P=None, shift=1)) == 1               # next-token shift needs prompt lengths
    assert lib.nat_prefix_pack(*pargs(rows=-1)) == 1
    assert lib.nat_prefix_pack(*pargs(src=None)) == 1
    assert lib.nat_prefix_pack(*pargs(tot=None)) == 1
    assert lib.nat_prefix_pack(*pargs(ids=fake)) == 1                      # gather pair incomplete


def test_loss_argument_errors(lib):
    fake = ctypes.c_void_p(256)
    f = ctypes.c_float
    def call(N_k=10, H=64, V=512, dtype=1, eps=0.2, hidden=fake, W=fake, ws=fake, ws_bytes=1 << 34):
        return lib.nat_loss_fwd_bwd(hidden, W, fake, fake, fake, fake, fake, N_k, H, V, dtype, f(eps), f(eps), f(1.0),
                                    fake, None, fake, fake, 0, ws, ws_bytes, None)
    assert call(dtype=7) == 4
    assert call(N_k=-1) == 1
    assert call(eps=-0.1) == 1
    assert call(H=0) == 2 and call(V=0) == 2
    assert call(H=100) == 2                      # bf16 kernels need H % 64 == 0
    assert call(W=None) == 1
    assert call(hidden=None) == 1
    assert call(ws_bytes=1024) == 3
    assert call(ws=None) == 3
    assert call(ws=ctypes.c_void_p(264)) == 1            # workspace not 256-byte aligned
    assert call(hidden=ctypes.c_void_p(260)) == 1        # 16-byte accesses on the caller's arrays
    assert call(W=ctypes.c_void_p(258)) == 1


def test_loss_kl_argument_errors(lib):
    fake = ctypes.c_void_p(256)
    f = ctypes.c_float
    def call(beta=0.1, kind=0, ref=fake, dtype=1, ws_bytes=1 << 34, N_k=10):
        return lib.nat_loss_fwd_bwd_kl(fake, fake, fake, fake, fake, fake, fake, N_k, 64, 512, dtype, f(0.2), f(0.2),
                                       f(1.0), ref, f(beta), kind, fake, None, None, None, None, fake, fake, 0, fake,
                                       ws_bytes, None)
    assert call(beta=-0.5) == 1
    assert call(beta=float("nan")) == 1
    assert call(kind=2) == 1 and call(kind=-1) == 1
    assert call(ref=None) == 1                     # a positive beta needs the reference log-probs
    assert call(dtype=9) == 4
    assert call(ws_bytes=64) == 3


def test_logp_fwd_argument_errors(lib):
    fake = ctypes.c_void_p(256)
    def call(N_k=10, H=64, V=512, dtype=1, hidden=fake, W=fake, logp=fake, ws=fake, ws_bytes=1 << 34):
        return lib.nat_logp_fwd(hidden, W, fake, N_k, H, V, dtype, logp, None, None, ws, ws_bytes, None)
    assert call(dtype=3) == 4
    assert call(N_k=-1) == 1
    assert call(H=100) == 2 and call(V=0) == 2
    assert call(hidden=None) == 1 and call(logp=None) == 1
    assert call(ws_bytes=100) == 3 and call(ws=None) == 3
    assert call(W=ctypes.c_void_p(264)) == 1
    assert call(N_k=0, hidden=None, ws=None) == 0            # nothing to do
    assert lib.nat_logp_workspace_bytes(1000, 4096, 151936, 1) < lib.nat_loss_workspace_bytes(1000, 4096, 151936, 1)
    assert lib.nat_logp_workspace_bytes(10, 100, 512, 1) == 0


def test_profile_interface(lib):
    n = lib.nat_profile_num_classes()
    names = [lib.nat_profile_class_name(i) for i in range(n)]
    assert b"logits_gemm" in names and b"dweight_gemm" in names and len(set(names)) == n
    ms = (ctypes.c_double * n)()
    cnt = (ctypes.c_int64 * n)()
    assert lib.nat_profile_collect(ms, cnt, n) == 0 and sum(cnt) == 0
    assert lib.nat_profile_collect(ms, cnt, 1) == 1
