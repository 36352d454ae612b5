"""MI355X-native fused LM-head log-probability objective (HIP, gfx950).

Thin Python binding over the C ABI declared in ``include/lmhead.h`` and, for the
token-adaptive KV-cache compression path, ``include/dynakv.h``.  PyTorch is
used only to own device memory and streams; every step of the path runs in the
library's HIP kernels.  There is no CPU fallback: if the shared library is
missing or no GPU is present, the compute entry points raise.
"""
from .binding import (
    LmheadError,
    LmheadDesc,
    library_path,
    load_library,
    make_desc,
    workspace_bytes,
    loss_workspace_bytes,
    validate_desc,
    lmhead_logprob_fwd,
    lmhead_logprob_fwd_multi,
    multi_workspace_bytes,
    lmhead_logprob_bwd,
    group_advantage,
    grpo_loss,
    grpo_loss_noalloc,
    flowrl_tb_loss,
    ce_loss,
    lmhead_check,
    lmhead_timing_enable,
    lmhead_timing_read,
    lmhead_probe_mfma,
    workspace_region,
    WS_NV, WS_ROW_SLOT, WS_TOK_C, WS_GATHERED_ID,
    EXPORTED_SYMBOLS,
)

from .dynakv import (
    DynakvDesc,
    make_kv_desc,
    dynakv_workspace_bytes,
    dynakv_validate_desc,
    dynakv_gate,
    dynakv_store,
    dynakv_reconstruct,
    dynakv_retain,
    dynakv_check,
    dynakv_bwd_workspace_bytes,
    dynakv_gate_bwd,
    FLAG_LITERAL_FLIP,
    FLAG_ACCUM_GRAD,
    DYNAKV_SYMBOLS,
)

__all__ = [
    "DynakvDesc", "make_kv_desc", "dynakv_workspace_bytes", "dynakv_validate_desc", "dynakv_gate",
    "dynakv_store", "dynakv_reconstruct", "dynakv_retain", "dynakv_check", "DYNAKV_SYMBOLS",
    "dynakv_bwd_workspace_bytes", "dynakv_gate_bwd", "FLAG_LITERAL_FLIP", "FLAG_ACCUM_GRAD",
    "LmheadError", "LmheadDesc", "library_path", "load_library", "make_desc",
    "workspace_bytes", "loss_workspace_bytes", "validate_desc",
    "lmhead_logprob_fwd", "lmhead_logprob_fwd_multi", "multi_workspace_bytes", "lmhead_logprob_bwd", "group_advantage", "grpo_loss", "grpo_loss_noalloc",
    "flowrl_tb_loss", "ce_loss", "lmhead_check", "lmhead_timing_enable", "lmhead_timing_read", "EXPORTED_SYMBOLS",
    "lmhead_probe_mfma", "workspace_region", "WS_NV", "WS_ROW_SLOT", "WS_TOK_C", "WS_GATHERED_ID",
]
