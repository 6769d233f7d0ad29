"""MI355X-native partial-token GRPO loss stage of NAT: thin Python binding over
the C-ABI library libnat_hip.so (hand-written HIP kernels for gfx950).

Every step of the path runs inside the library; this package only marshals
arguments (torch tensors -> device pointers, the current HIP stream)."""
from .binding import (  # noqa: F401
    NatError, SelectParams, FULL, URS, RPC, DET, DTYPE_F32, DTYPE_BF16, KL_LOG_RATIO, KL_NONNEG,
    DIAG_BAD_ID, DIAG_SHIFT_RANGE, DIAG_CLIPPED, DIAG_NONZERO_ADV, DIAG_WORDS,
    load_library, library_path, status_string, mask_words,
    nat_advantage, nat_select, nat_compact, nat_compact_static, nat_loss_fwd_bwd,
    nat_select_schedule, nat_select_poisson, nat_compact_pi, nat_prefix_pack, nat_loss_fwd_bwd_kl, nat_logp_fwd, logp_workspace_bytes, logp_workspace_min_bytes,
    compact_workspace_bytes, loss_workspace_bytes, loss_workspace_min_bytes,
    profile_enable, profile_collect, probe_mfma_scratch_bytes, nat_probe_mfma_bf16, nat_probe_copy,
)
