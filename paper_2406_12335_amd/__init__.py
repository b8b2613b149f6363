"""MI355X-native value-aware token pruning (VATP) hot path: HIP kernels behind a C ABI.

`binding` mirrors the C entry points one to one; `runner.PrunedKVCache` only owns the
device buffers of a pruned per-head KV cache and calls the entry points in order.
"""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    CALL_DECODE_ATTEND_STEP, CALL_DECODE_PRUNE_STEP, CALL_DECODE_STEP, CALL_PREFILL_SCORE_WINDOW, CALL_PREFILL_SCORE, CALL_SELECT_COMPACT, NORM_L1, NORM_L2, NORM_LINF, NORM_NONE, VATP_BF16, VATP_F32, Params,
    VatpError,
    load, strerror, vatp_create, vatp_decode_attend_step, vatp_decode_prune_step, vatp_decode_prune_step_static, vatp_decode_prune_step_window, vatp_decode_step, vatp_destroy, vatp_prefill_score, vatp_prefill_score_lse, vatp_prefill_score_window, vatp_select_compact,
    vatp_select_compact_window,
    vatp_validate, vatp_workspace_bytes,
)
