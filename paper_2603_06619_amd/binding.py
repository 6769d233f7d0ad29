"""ctypes binding of include/nat.h.  Argument marshalling only."""
import ctypes
import os

import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libnat_hip.so"
_lib = None

FULL, URS, RPC, DET = 0, 1, 2, 3
DTYPE_F32, DTYPE_BF16 = 0, 1
KL_LOG_RATIO, KL_NONNEG = 0, 1
DIAG_BAD_ID, DIAG_SHIFT_RANGE, DIAG_CLIPPED, DIAG_NONZERO_ADV, DIAG_WORDS = 0, 1, 2, 3, 4


class NatError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where} failed: {status_string(status)} ({status})")


class _CSelectParams(ctypes.Structure):
    _fields_ = [("scheme", ctypes.c_int32), ("min_cut", ctypes.c_int32), ("p", ctypes.c_double),
                ("trunc_frac", ctypes.c_double), ("seed", ctypes.c_uint64), ("step", ctypes.c_uint32),
                ("rollout_id_base", ctypes.c_int32), ("d_scheme_per_rollout", ctypes.c_void_p),
                ("d_drop_zero_adv", ctypes.c_void_p)]


class SelectParams:
    """Selection parameters of nat_select / nat_compact (see nat_select_params in nat.h)."""

    def __init__(self, scheme, p=1.0, min_cut=1, trunc_frac=1.0, seed=0, step=0, rollout_id_base=0,
                 scheme_per_rollout=None, drop_zero_adv=None):
        self.scheme, self.p, self.min_cut, self.trunc_frac = scheme, p, min_cut, trunc_frac
        self.seed, self.step, self.rollout_id_base = seed, step, rollout_id_base
        self.scheme_per_rollout = scheme_per_rollout      # int32 device tensor [B] or None
        self.drop_zero_adv = drop_zero_adv                # float32 device tensor [B] of advantages or None

    def _c(self):
        spr = self.scheme_per_rollout
        if spr is not None:
            _check(spr, torch.int32, "scheme_per_rollout")
        return _CSelectParams(int(self.scheme), int(self.min_cut), float(self.p), float(self.trunc_frac),
                              int(self.seed) & (2 ** 64 - 1), int(self.step) & 0xFFFFFFFF, int(self.rollout_id_base),
                              spr.data_ptr() if spr is not None else None,
                              _check(self.drop_zero_adv, torch.float32, "drop_zero_adv").data_ptr()
                              if self.drop_zero_adv is not None else None)


def library_path():
    # NAT_HIP_LIBRARY selects another build of the same library (A/B timing of kernel variants)
    return os.environ.get("NAT_HIP_LIBRARY") or os.path.join(_PKG_DIR, _LIB_NAME)


def load_library():
    """Load the built library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is missing: build it with `python -m paper_2603_06619_amd.build`")
    lib = ctypes.CDLL(path)
    vp, i32, i64, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
    pp = ctypes.POINTER(_CSelectParams)
    lib.nat_status_string.restype = ctypes.c_char_p
    lib.nat_status_string.argtypes = [i32]
    lib.nat_mask_words.restype = i64
    lib.nat_mask_words.argtypes = [i64]
    lib.nat_advantage.restype = i32
    lib.nat_advantage.argtypes = [vp, i32, i32, f32, vp, vp]
    lib.nat_select.restype = i32
    lib.nat_select.argtypes = [pp, vp, i32, i64, vp, vp, vp]
    lib.nat_compact_workspace_bytes.restype = sz
    lib.nat_compact_workspace_bytes.argtypes = [i64]
    lib.nat_compact.restype = i32
    lib.nat_compact.argtypes = [pp, i32, vp, vp, i32, i64, i64, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32,
                                vp, vp, vp, vp, vp, sz, vp]
    lib.nat_compact_static.restype = i32
    lib.nat_compact_static.argtypes = [pp, i32, vp, vp, i32, i64, i64, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32,
                                       vp, vp, vp, vp, vp]
    lib.nat_select_schedule.restype = i32
    lib.nat_select_schedule.argtypes = [pp, vp, vp, i32, i64, vp, vp, vp, vp]
    lib.nat_select_poisson.restype = i32
    lib.nat_select_poisson.argtypes = [pp, vp, vp, i32, i64, vp, vp]
    lib.nat_compact_pi.restype = i32
    lib.nat_compact_pi.argtypes = [i32, vp, vp, vp, i32, i64, i64, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32,
                                   vp, vp, vp, vp, vp, sz, vp]
    lib.nat_prefix_pack.restype = i32
    lib.nat_prefix_pack.argtypes = [vp, vp, vp, i32, i32, i64, i64, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    for name in ("nat_loss_workspace_bytes", "nat_loss_workspace_min_bytes"):
        getattr(lib, name).restype = sz
        getattr(lib, name).argtypes = [i32, i32, i32, i32]
    lib.nat_loss_fwd_bwd.restype = i32
    lib.nat_loss_fwd_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, f32, f32, f32,
                                     vp, vp, vp, vp, i32, vp, sz, vp]
    lib.nat_loss_fwd_bwd_kl.restype = i32
    lib.nat_loss_fwd_bwd_kl.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, f32, f32, f32,
                                        vp, f32, i32, vp, vp, vp, vp, vp, vp, vp, i32, vp, sz, vp]
    for name in ("nat_logp_workspace_bytes", "nat_logp_workspace_min_bytes"):
        getattr(lib, name).restype = sz
        getattr(lib, name).argtypes = [i32, i32, i32, i32]
    lib.nat_logp_fwd.restype = i32
    lib.nat_logp_fwd.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, sz, vp]
    lib.nat_probe_mfma_scratch_bytes.restype = sz
    lib.nat_probe_mfma_scratch_bytes.argtypes = []
    lib.nat_probe_mfma_bf16.restype = i32
    lib.nat_probe_mfma_bf16.argtypes = [i32, i32, vp, ctypes.POINTER(ctypes.c_double), vp]
    lib.nat_probe_copy.restype = i32
    lib.nat_probe_copy.argtypes = [vp, vp, sz, vp]
    lib.nat_profile_num_classes.restype = i32
    lib.nat_profile_class_name.restype = ctypes.c_char_p
    lib.nat_profile_class_name.argtypes = [i32]
    lib.nat_profile_enable.restype = i32
    lib.nat_profile_enable.argtypes = [i32]
    lib.nat_profile_collect.restype = i32
    lib.nat_profile_collect.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64), i32]
    _lib = lib
    return lib


def status_string(status):
    return load_library().nat_status_string(int(status)).decode()


def _check(t, dtype, name):
    if not isinstance(t, torch.Tensor) or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name}: expected a contiguous {dtype} tensor")
    return t


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _raise(status, where):
    if status != 0:
        raise NatError(status, where)


def _dtype_code(t):
    if t.dtype == torch.float32:
        return DTYPE_F32
    if t.dtype == torch.bfloat16:
        return DTYPE_BF16
    raise TypeError("hidden / W must be float32 or bfloat16")


def mask_words(N):
    return int(load_library().nat_mask_words(int(N)))


def compact_workspace_bytes(N):
    return int(load_library().nat_compact_workspace_bytes(int(N)))


def loss_workspace_bytes(N_k, H, V, dtype):
    return int(load_library().nat_loss_workspace_bytes(int(N_k), int(H), int(V), int(dtype)))


def loss_workspace_min_bytes(N_k, H, V, dtype):
    return int(load_library().nat_loss_workspace_min_bytes(int(N_k), int(H), int(V), int(dtype)))


def nat_advantage(rewards, P, G, eps_adv, adv_out):
    _check(rewards, torch.float32, "rewards")
    _check(adv_out, torch.float32, "adv_out")
    _raise(load_library().nat_advantage(_ptr(rewards), P, G, eps_adv, _ptr(adv_out), _stream()), "nat_advantage")


def nat_select(params, cu_seqlens, B, N, cut_len_out, mask_bits_out):
    _check(cu_seqlens, torch.int64, "cu_seqlens")
    _check(cut_len_out, torch.int32, "cut_len_out")
    _check(mask_bits_out, torch.int32, "mask_bits_out")
    c = params._c()
    _raise(load_library().nat_select(ctypes.byref(c), _ptr(cu_seqlens), B, N, _ptr(cut_len_out),
                                     _ptr(mask_bits_out), _stream()), "nat_select")


def _kept_cap(kept_cap, kept_idx):
    return int(kept_idx.numel() if kept_cap is None and kept_idx is not None else (kept_cap or 0))


def nat_compact(params, n_rollouts_global, mask_bits, cu_seqlens, B, N, kept_idx, kept_seq, kept_w, cu_kept,
                n_kept, h_n_kept, workspace, hidden=None, hidden_k=None, ids=None, ids_k=None,
                old_logp=None, old_logp_k=None, kept_cap=None):
    """kept_cap: capacity of the per-kept-token outputs; default: the length of kept_idx."""
    c = params._c()
    H = hidden.shape[1] if hidden is not None else 0
    dt = _dtype_code(hidden) if hidden is not None else DTYPE_F32
    _raise(load_library().nat_compact(
        ctypes.byref(c), n_rollouts_global, _ptr(mask_bits), _ptr(cu_seqlens), B, N, _kept_cap(kept_cap, kept_idx),
        _ptr(kept_idx), _ptr(kept_seq),
        _ptr(kept_w), _ptr(cu_kept), _ptr(n_kept), _ptr(h_n_kept), _ptr(hidden), _ptr(hidden_k), H, dt,
        _ptr(ids), _ptr(ids_k), _ptr(old_logp), _ptr(old_logp_k), _ptr(workspace),
        workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream()), "nat_compact")


def nat_compact_static(params, n_rollouts_global, mask_bits, cu_seqlens, B, N, kept_idx, kept_seq, kept_w, cu_kept,
                       n_kept, h_n_kept, hidden=None, hidden_k=None, ids=None, ids_k=None,
                       old_logp=None, old_logp_k=None, kept_cap=None):
    """nat_compact without a workspace argument (the library's resident scratch); allocates nothing."""
    c = params._c()
    H = hidden.shape[1] if hidden is not None else 0
    dt = _dtype_code(hidden) if hidden is not None else DTYPE_F32
    _raise(load_library().nat_compact_static(
        ctypes.byref(c), n_rollouts_global, _ptr(mask_bits), _ptr(cu_seqlens), B, N, _kept_cap(kept_cap, kept_idx),
        _ptr(kept_idx), _ptr(kept_seq), _ptr(kept_w), _ptr(cu_kept), _ptr(n_kept), _ptr(h_n_kept), _ptr(hidden),
        _ptr(hidden_k), H, dt, _ptr(ids), _ptr(ids_k), _ptr(old_logp), _ptr(old_logp_k), _stream()),
        "nat_compact_static")


def nat_select_schedule(params, weights, cu_seqlens, B, N, cut_len_out, mask_bits_out, pi_out):
    _check(cu_seqlens, torch.int64, "cu_seqlens")
    _check(weights, torch.int32, "weights")          # the 32 bits are read as unsigned
    _check(cut_len_out, torch.int32, "cut_len_out")
    _check(mask_bits_out, torch.int32, "mask_bits_out")
    _check(pi_out, torch.float64, "pi_out")
    c = params._c()
    _raise(load_library().nat_select_schedule(ctypes.byref(c), _ptr(weights), _ptr(cu_seqlens), B, N,
                                              _ptr(cut_len_out), _ptr(mask_bits_out), _ptr(pi_out), _stream()),
           "nat_select_schedule")


def nat_select_poisson(params, pi, cu_seqlens, B, N, mask_bits_out):
    _check(cu_seqlens, torch.int64, "cu_seqlens")
    _check(pi, torch.float64, "pi")
    _check(mask_bits_out, torch.int32, "mask_bits_out")
    c = params._c()
    _raise(load_library().nat_select_poisson(ctypes.byref(c), _ptr(pi), _ptr(cu_seqlens), B, N,
                                             _ptr(mask_bits_out), _stream()), "nat_select_poisson")


def nat_compact_pi(n_rollouts_global, mask_bits, pi, cu_seqlens, B, N, kept_idx, kept_seq, kept_w, cu_kept,
                   n_kept, h_n_kept, workspace, hidden=None, hidden_k=None, ids=None, ids_k=None,
                   old_logp=None, old_logp_k=None, kept_cap=None):
    _check(pi, torch.float64, "pi")
    H = hidden.shape[1] if hidden is not None else 0
    dt = _dtype_code(hidden) if hidden is not None else DTYPE_F32
    _raise(load_library().nat_compact_pi(
        n_rollouts_global, _ptr(mask_bits), _ptr(pi), _ptr(cu_seqlens), B, N, _kept_cap(kept_cap, kept_idx),
        _ptr(kept_idx), _ptr(kept_seq),
        _ptr(kept_w), _ptr(cu_kept), _ptr(n_kept), _ptr(h_n_kept), _ptr(hidden), _ptr(hidden_k), H, dt,
        _ptr(ids), _ptr(ids_k), _ptr(old_logp), _ptr(old_logp_k), _ptr(workspace),
        workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream()), "nat_compact_pi")


def nat_prefix_pack(prompt_len, cu_seqlens, cut_len, B, next_token_shift, rows_cap, kept_cap, cu_packed, cu_loss,
                    src_idx, position_ids, loss_row, totals, h_totals, input_ids=None, input_ids_packed=None):
    _check(cu_seqlens, torch.int64, "cu_seqlens")
    _check(cut_len, torch.int32, "cut_len")
    _raise(load_library().nat_prefix_pack(
        _ptr(prompt_len), _ptr(cu_seqlens), _ptr(cut_len), B, int(next_token_shift), int(rows_cap), int(kept_cap),
        _ptr(cu_packed), _ptr(cu_loss), _ptr(src_idx), _ptr(position_ids), _ptr(loss_row), _ptr(totals),
        _ptr(h_totals), _ptr(input_ids), _ptr(input_ids_packed), _stream()), "nat_prefix_pack")


def nat_loss_fwd_bwd(hidden_k, W, ids_k, old_logp_k, adv, kept_seq, kept_w, N_k, eps_lo, eps_hi, grad_scale,
                     loss_out, logp_out, dH_out, dW_out, accumulate_dw, workspace):
    V, H = W.shape
    _raise(load_library().nat_loss_fwd_bwd(
        _ptr(hidden_k), _ptr(W), _ptr(ids_k), _ptr(old_logp_k), _ptr(adv), _ptr(kept_seq), _ptr(kept_w),
        N_k, H, V, _dtype_code(W), eps_lo, eps_hi, grad_scale, _ptr(loss_out), _ptr(logp_out), _ptr(dH_out),
        _ptr(dW_out), int(accumulate_dw), _ptr(workspace),
        workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream()), "nat_loss_fwd_bwd")


def nat_loss_fwd_bwd_kl(hidden_k, W, ids_k, old_logp_k, adv, kept_seq, kept_w, N_k, eps_lo, eps_hi, grad_scale,
                        ref_logp_k, beta_kl, kl_kind, loss_out, logp_out, kl_out, entropy_out, dH_out, dW_out,
                        accumulate_dw, workspace, diag_out=None):
    V, H = W.shape
    _raise(load_library().nat_loss_fwd_bwd_kl(
        _ptr(hidden_k), _ptr(W), _ptr(ids_k), _ptr(old_logp_k), _ptr(adv), _ptr(kept_seq), _ptr(kept_w),
        N_k, H, V, _dtype_code(W), eps_lo, eps_hi, grad_scale, _ptr(ref_logp_k), float(beta_kl), int(kl_kind),
        _ptr(loss_out), _ptr(logp_out), _ptr(kl_out), _ptr(entropy_out), _ptr(diag_out), _ptr(dH_out), _ptr(dW_out),
        int(accumulate_dw), _ptr(workspace),
        workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream()),
        "nat_loss_fwd_bwd_kl")


def logp_workspace_bytes(N_k, H, V, dtype):
    return int(load_library().nat_logp_workspace_bytes(int(N_k), int(H), int(V), int(dtype)))


def logp_workspace_min_bytes(N_k, H, V, dtype):
    return int(load_library().nat_logp_workspace_min_bytes(int(N_k), int(H), int(V), int(dtype)))


def nat_logp_fwd(hidden_k, W, ids_k, N_k, logp_out, entropy_out, workspace, diag_out=None):
    V, H = W.shape
    _raise(load_library().nat_logp_fwd(
        _ptr(hidden_k), _ptr(W), _ptr(ids_k), N_k, H, V, _dtype_code(W), _ptr(logp_out), _ptr(entropy_out),
        _ptr(diag_out), _ptr(workspace), workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream()),
        "nat_logp_fwd")


def probe_mfma_scratch_bytes():
    return int(load_library().nat_probe_mfma_scratch_bytes())


def nat_probe_mfma_bf16(random_operands, iters, scratch):
    """Launches the matrix-core probe on the current stream; returns the flops of the launch."""
    flops = ctypes.c_double(0.0)
    _raise(load_library().nat_probe_mfma_bf16(int(bool(random_operands)), int(iters), _ptr(scratch),
                                              ctypes.byref(flops), _stream()), "nat_probe_mfma_bf16")
    return flops.value


def nat_probe_copy(dst, src, nbytes):
    _raise(load_library().nat_probe_copy(_ptr(dst), _ptr(src), int(nbytes), _stream()), "nat_probe_copy")


def profile_enable(on):
    _raise(load_library().nat_profile_enable(int(bool(on))), "nat_profile_enable")


def profile_collect():
    """Returns {class name: (milliseconds, launches)} accumulated since the last call."""
    lib = load_library()
    n = lib.nat_profile_num_classes()
    ms = (ctypes.c_double * n)()
    cnt = (ctypes.c_int64 * n)()
    _raise(lib.nat_profile_collect(ms, cnt, n), "nat_profile_collect")
    return {lib.nat_profile_class_name(i).decode(): (ms[i], cnt[i]) for i in range(n)}
