"""Buffer plumbing around the four library calls: allocates outputs and
workspaces with torch and issues advantage -> select -> compact -> loss on the
current stream.  No arithmetic of the method happens here."""
import torch

from . import binding as nb


class LossStage:
    def __init__(self, device="cuda:0"):
        self.device = torch.device(device)
        self._ws = {}
        self.h_n_kept = torch.zeros(1, dtype=torch.int32).pin_memory()
        self.h_totals = torch.zeros(2, dtype=torch.int32).pin_memory()

    def _buf(self, key, nbytes):
        t = self._ws.get(key)
        if t is None or t.numel() < nbytes:
            t = torch.empty(int(nbytes), dtype=torch.uint8, device=self.device)
            self._ws[key] = t
        return t

    def advantage(self, rewards, P, G, eps_adv=1e-6):
        adv = torch.empty(P * G, dtype=torch.float32, device=self.device)
        nb.nat_advantage(rewards, P, G, eps_adv, adv)
        return adv

    def select_compact(self, params, cu_seqlens, B, N, n_rollouts_global=None, hidden=None, ids=None, old_logp=None,
                       schedule_weights=None, poisson_pi=None):
        """Returns dict with cut_len, mask_bits, kept_idx/seq/w (length N, first n_kept valid), cu_kept,
        n_kept (host int, read after a stream sync) and the gathered rows when inputs are given.
        schedule_weights (int32 [N], read as unsigned) selects nat_select_schedule, poisson_pi (float64 [N])
        nat_select_poisson; both then weight through nat_compact_pi and the dict also holds `pi`."""
        dev = self.device
        out = dict(cut_len=torch.empty(B, dtype=torch.int32, device=dev),
                   mask_bits=torch.empty(max(nb.mask_words(N), 1), dtype=torch.int32, device=dev),
                   kept_idx=torch.empty(max(N, 1), dtype=torch.int32, device=dev),
                   kept_seq=torch.empty(max(N, 1), dtype=torch.int32, device=dev),
                   kept_w=torch.empty(max(N, 1), dtype=torch.float32, device=dev),
                   cu_kept=torch.empty(B + 1, dtype=torch.int32, device=dev),
                   n_kept_dev=torch.empty(1, dtype=torch.int32, device=dev))
        if schedule_weights is not None:
            out["pi"] = torch.empty(max(N, 1), dtype=torch.float64, device=dev)
            nb.nat_select_schedule(params, schedule_weights, cu_seqlens, B, N, out["cut_len"], out["mask_bits"],
                                   out["pi"])
        elif poisson_pi is not None:
            out["pi"] = poisson_pi
            out["cut_len"] = None
            nb.nat_select_poisson(params, poisson_pi, cu_seqlens, B, N, out["mask_bits"])
        else:
            nb.nat_select(params, cu_seqlens, B, N, out["cut_len"], out["mask_bits"])
        if hidden is not None:
            out["hidden_k"] = torch.empty((max(N, 1), hidden.shape[1]), dtype=hidden.dtype, device=dev)
        if ids is not None:
            out["ids_k"] = torch.empty(max(N, 1), dtype=torch.int32, device=dev)
        if old_logp is not None:
            out["old_logp_k"] = torch.empty(max(N, 1), dtype=torch.float32, device=dev)
        ws = self._buf("compact", nb.compact_workspace_bytes(N))
        nB = n_rollouts_global if n_rollouts_global is not None else B
        if "pi" in out:
            nb.nat_compact_pi(nB, out["mask_bits"], out["pi"], cu_seqlens, B, N, out["kept_idx"], out["kept_seq"],
                              out["kept_w"], out["cu_kept"], out["n_kept_dev"], self.h_n_kept, ws, hidden,
                              out.get("hidden_k"), ids, out.get("ids_k"), old_logp, out.get("old_logp_k"))
        else:
            nb.nat_compact(params, nB, out["mask_bits"], cu_seqlens, B, N, out["kept_idx"], out["kept_seq"],
                           out["kept_w"], out["cu_kept"], out["n_kept_dev"], self.h_n_kept, ws, hidden,
                           out.get("hidden_k"), ids, out.get("ids_k"), old_logp, out.get("old_logp_k"))
        torch.cuda.current_stream().synchronize()        # the one documented read-back: n_kept
        out["n_kept"] = int(self.h_n_kept[0])
        return out

    def prefix_pack(self, prompt_len, cu_seqlens, cut_len, B, N, rows_cap, next_token_shift=1, input_ids=None):
        """Truncated batch (prompt + kept prefix per rollout).  rows_cap: an upper bound on its rows, e.g. the
        rows of the full input.  Returns the device arrays and, after one stream sync, total and max_len."""
        dev = self.device
        i32 = lambda n: torch.empty(max(int(n), 1), dtype=torch.int32, device=dev)
        out = dict(cu_packed=i32(B + 1), cu_loss=i32(B + 1), src_idx=i32(rows_cap), position_ids=i32(rows_cap),
                   loss_row=i32(N), totals=i32(2))
        if input_ids is not None:
            out["input_ids_packed"] = i32(rows_cap)
        nb.nat_prefix_pack(prompt_len, cu_seqlens, cut_len, B, next_token_shift, rows_cap, N, out["cu_packed"],
                           out["cu_loss"], out["src_idx"], out["position_ids"], out["loss_row"], out["totals"],
                           self.h_totals, input_ids, out.get("input_ids_packed"))
        torch.cuda.current_stream().synchronize()
        out["total"], out["max_len"] = int(self.h_totals[0]), int(self.h_totals[1])
        return out

    def logp(self, hidden_k, W, ids_k, N_k, want_entropy=False, ws_bytes=None, want_diag=False):
        """Forward pass alone: log-probs (and entropies) of the given tokens."""
        dev = self.device
        V, H = W.shape
        dt = nb.DTYPE_BF16 if W.dtype == torch.bfloat16 else nb.DTYPE_F32
        if ws_bytes is None:
            ws_bytes = nb.logp_workspace_bytes(N_k, H, V, dt)
        ws = self._buf("loss", max(ws_bytes, 256))[:max(ws_bytes, 256)]
        out = dict(logp=torch.empty(max(N_k, 1), dtype=torch.float32, device=dev),
                   entropy=torch.empty(max(N_k, 1), dtype=torch.float32, device=dev) if want_entropy else None,
                   diag=torch.empty(nb.DIAG_WORDS, dtype=torch.int32, device=dev) if want_diag else None)
        nb.nat_logp_fwd(hidden_k, W, ids_k, N_k, out["logp"], out["entropy"], ws, out["diag"])
        return out

    def loss(self, hidden_k, W, ids_k, old_logp_k, adv, kept_seq, kept_w, N_k, eps_lo=0.2, eps_hi=0.2,
             grad_scale=1.0, dW=None, accumulate_dw=False, ws_bytes=None, want_logp=True,
             ref_logp_k=None, beta_kl=0.0, kl_kind=nb.KL_LOG_RATIO, want_kl=False, want_entropy=False,
             want_diag=False):
        dev = self.device
        V, H = W.shape
        dt = nb.DTYPE_BF16 if W.dtype == torch.bfloat16 else nb.DTYPE_F32
        if ws_bytes is None:
            ws_bytes = nb.loss_workspace_bytes(N_k, H, V, dt)
        ws = self._buf("loss", max(ws_bytes, 256))[:max(ws_bytes, 256)]
        out = dict(loss=torch.empty(1, dtype=torch.float32, device=dev),
                   logp=torch.empty(max(N_k, 1), dtype=torch.float32, device=dev) if want_logp else None,
                   dH=torch.empty((max(N_k, 1), H), dtype=W.dtype, device=dev),
                   dW=dW if dW is not None else torch.empty((V, H), dtype=torch.float32, device=dev))
        if ref_logp_k is None and not want_kl and not want_entropy and not want_diag:
            nb.nat_loss_fwd_bwd(hidden_k, W, ids_k, old_logp_k, adv, kept_seq, kept_w, N_k, eps_lo, eps_hi, grad_scale,
                                out["loss"], out["logp"], out["dH"], out["dW"], accumulate_dw, ws)
            return out
        f32 = lambda: torch.empty(max(N_k, 1), dtype=torch.float32, device=dev)
        out["kl"] = f32() if want_kl else None
        out["entropy"] = f32() if want_entropy else None
        out["diag"] = torch.empty(nb.DIAG_WORDS, dtype=torch.int32, device=dev) if want_diag else None
        nb.nat_loss_fwd_bwd_kl(hidden_k, W, ids_k, old_logp_k, adv, kept_seq, kept_w, N_k, eps_lo, eps_hi, grad_scale,
                               ref_logp_k, beta_kl, kl_kind, out["loss"], out["logp"], out["kl"], out["entropy"],
                               out["dH"], out["dW"], accumulate_dw, ws, out["diag"])
        return out
