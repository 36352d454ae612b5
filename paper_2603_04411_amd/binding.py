"""ctypes binding of liblmhead.so: argument marshalling only.

Every function has the name and argument order of its C counterpart in
``include/lmhead.h``.  Tensors are torch CUDA (ROCm) tensors; the binding passes
their device pointers and the current stream and raises ``LmheadError`` on a
negative status.  Nothing is computed here.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))

EXPORTED_SYMBOLS = [
    "lmhead_abi_version", "lmhead_workspace_bytes", "lmhead_validate_desc",
    "lmhead_logprob_fwd", "lmhead_logprob_bwd", "lmhead_multi_workspace_bytes", "lmhead_logprob_fwd_multi",
    "group_advantage",
    "lmhead_loss_workspace_bytes", "grpo_loss", "grpo_loss_noalloc", "flowrl_tb_loss", "ce_loss", "lmhead_check",
    "lmhead_timing_enable", "lmhead_timing_read", "lmhead_workspace_region", "lmhead_probe_mfma",
]

ERRORS = {
    -1: "LMHEAD_E_NULL", -2: "LMHEAD_E_SHAPE", -3: "LMHEAD_E_DTYPE", -4: "LMHEAD_E_ALIGN",
    -5: "LMHEAD_E_WORKSPACE", -6: "LMHEAD_E_RANGE", -7: "LMHEAD_E_HIP",
}

LMHEAD_F32 = 0
LMHEAD_BF16 = 1
FLAG_ACCUM_DW = 1 << 1
FLAG_FP8_LOGITS = 1 << 2
FLAG_DH_BF16 = 1 << 3


class LmheadError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {ERRORS.get(code, code)}")


class LmheadDesc(C.Structure):
    _fields_ = [
        ("P", C.c_int32), ("G", C.c_int32), ("T", C.c_int32),
        ("d", C.c_int32), ("V", C.c_int32),
        ("dtype", C.c_int32), ("vocab_chunk", C.c_int32), ("fp8_exp_h", C.c_int32),
        ("ldH", C.c_int64), ("ldW", C.c_int64),
        ("flags", C.c_uint32), ("fp8_exp_w", C.c_int32),
    ]


_lib = None


def library_path() -> str:
    return os.path.join(HERE, "liblmhead.so")


def load_library():
    """Loads liblmhead.so (built by ``paper_2603_04411_amd.build``); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} not found: build it with `python -m paper_2603_04411_amd.build` (there is no fallback path)")
    lib = C.CDLL(path)
    vp, i32, f32, sz = C.c_void_p, C.c_int32, C.c_float, C.c_size_t
    dp = C.POINTER(LmheadDesc)
    lib.lmhead_abi_version.restype = C.c_int
    lib.lmhead_abi_version.argtypes = []
    lib.lmhead_workspace_bytes.restype = sz
    lib.lmhead_workspace_bytes.argtypes = [dp]
    lib.lmhead_validate_desc.restype = C.c_int
    lib.lmhead_validate_desc.argtypes = [dp]
    lib.lmhead_logprob_fwd.restype = C.c_int
    lib.lmhead_logprob_fwd.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.lmhead_multi_workspace_bytes.restype = sz
    lib.lmhead_multi_workspace_bytes.argtypes = [dp, i32]
    lib.lmhead_logprob_fwd_multi.restype = C.c_int
    lib.lmhead_logprob_fwd_multi.argtypes = [dp, vp, C.POINTER(vp), i32, vp, vp, C.POINTER(vp), vp, vp, vp, vp, vp,
                                             sz, vp]
    lib.lmhead_logprob_bwd.restype = C.c_int
    lib.lmhead_logprob_bwd.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.group_advantage.restype = C.c_int
    lib.group_advantage.argtypes = [vp, i32, i32, f32, i32, vp, vp]
    lib.lmhead_loss_workspace_bytes.restype = sz
    lib.lmhead_loss_workspace_bytes.argtypes = [i32, i32, i32]
    lib.grpo_loss.restype = C.c_int
    lib.grpo_loss.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, f32, f32, f32, i32, vp, vp, vp, vp, sz, vp]
    lib.grpo_loss_noalloc.restype = C.c_int
    lib.grpo_loss_noalloc.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, f32, f32, f32, i32, vp, vp, vp, vp]
    lib.flowrl_tb_loss.restype = C.c_int
    lib.flowrl_tb_loss.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, f32, vp, vp, vp, vp, vp, sz, vp]
    lib.ce_loss.restype = C.c_int
    lib.ce_loss.argtypes = [vp, vp, i32, i32, vp, vp, vp, sz, vp]
    lib.lmhead_check.restype = C.c_int
    lib.lmhead_check.argtypes = [vp, vp]
    lib.lmhead_workspace_region.restype = C.c_int
    lib.lmhead_workspace_region.argtypes = [dp, i32, i32, C.POINTER(sz), C.POINTER(sz)]
    lib.lmhead_probe_mfma.restype = C.c_int
    lib.lmhead_probe_mfma.argtypes = [vp, sz, vp, sz, i32, i32, vp]
    lib.lmhead_timing_enable.restype = C.c_int
    lib.lmhead_timing_enable.argtypes = [C.c_int]
    lib.lmhead_timing_read.restype = C.c_int
    lib.lmhead_timing_read.argtypes = [C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    _lib = lib
    return lib


def make_desc(P, G, T, d, V, dtype, vocab_chunk=0, ldH=None, ldW=None, flags=0, fp8_exp_h=0,
              fp8_exp_w=0) -> LmheadDesc:
    code = {"bf16": LMHEAD_BF16, "f32": LMHEAD_F32}.get(dtype, dtype)
    return LmheadDesc(P=P, G=G, T=T, d=d, V=V, dtype=code, vocab_chunk=vocab_chunk, fp8_exp_h=fp8_exp_h,
                      ldH=d if ldH is None else ldH, ldW=d if ldW is None else ldW,
                      flags=flags, fp8_exp_w=fp8_exp_w)


def workspace_bytes(desc: LmheadDesc) -> int:
    return int(load_library().lmhead_workspace_bytes(C.byref(desc)))


def loss_workspace_bytes(P: int, G: int, T: int) -> int:
    return int(load_library().lmhead_loss_workspace_bytes(P, G, T))


def validate_desc(desc: LmheadDesc) -> int:
    return int(load_library().lmhead_validate_desc(C.byref(desc)))


WS_NV, WS_ROW_SLOT, WS_TOK_C, WS_GATHERED_ID = 0, 1, 2, 3


def workspace_region(desc: LmheadDesc, npol: int, which: int):
    """(byte offset, bytes) of one of the integer index regions a forward call leaves in its workspace."""
    off, nbytes = C.c_size_t(0), C.c_size_t(0)
    _check(load_library().lmhead_workspace_region(C.byref(desc), npol, which, C.byref(off), C.byref(nbytes)),
           "lmhead_workspace_region")
    return off.value, nbytes.value


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    return t.data_ptr()


def _stream() -> Optional[int]:
    import torch
    return torch.cuda.current_stream().cuda_stream or None


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise LmheadError(rc, where)


def lmhead_logprob_fwd(desc, H, W, tok, lens, logp, lse, entropy, mask, cu_len, ws) -> None:
    rc = load_library().lmhead_logprob_fwd(
        C.byref(desc), _ptr(H), _ptr(W), _ptr(tok), _ptr(lens), _ptr(logp), _ptr(lse), _ptr(entropy),
        _ptr(mask), _ptr(cu_len), _ptr(ws), ws.numel() * ws.element_size(), _stream())
    _check(rc, "lmhead_logprob_fwd")


def multi_workspace_bytes(desc: LmheadDesc, npol: int) -> int:
    return int(load_library().lmhead_multi_workspace_bytes(C.byref(desc), npol))


def lmhead_logprob_fwd_multi(desc, H, Ws, tok, lens, logps, lse, entropy, mask, cu_len, ws) -> None:
    """Ws / logps: sequences of npol device tensors (weight matrices / log-prob outputs)."""
    npol = len(Ws)
    if len(logps) != npol:
        raise ValueError("one log-prob output per weight matrix")
    w_arr = (C.c_void_p * npol)(*[_ptr(t) for t in Ws])
    lp_arr = (C.c_void_p * npol)(*[_ptr(t) for t in logps])
    rc = load_library().lmhead_logprob_fwd_multi(
        C.byref(desc), _ptr(H), w_arr, npol, _ptr(tok), _ptr(lens), lp_arr, _ptr(lse), _ptr(entropy),
        _ptr(mask), _ptr(cu_len), _ptr(ws), ws.numel() * ws.element_size(), _stream())
    _check(rc, "lmhead_logprob_fwd_multi")


def lmhead_logprob_bwd(desc, H, W, tok, lens, lse, g_logp, dH, dW, ws) -> None:
    rc = load_library().lmhead_logprob_bwd(
        C.byref(desc), _ptr(H), _ptr(W), _ptr(tok), _ptr(lens), _ptr(lse), _ptr(g_logp), _ptr(dH), _ptr(dW),
        _ptr(ws), ws.numel() * ws.element_size(), _stream())
    _check(rc, "lmhead_logprob_bwd")


def group_advantage(reward, P, G, eps, ddof, adv) -> None:
    _check(load_library().group_advantage(_ptr(reward), P, G, eps, ddof, _ptr(adv), _stream()), "group_advantage")


def grpo_loss(logp, logp_old, logp_ref, adv, lens, P, G, T, clip_lo, clip_hi, kl_coef, agg_mode,
              loss, g_logp, stats, ws) -> None:
    rc = load_library().grpo_loss(
        _ptr(logp), _ptr(logp_old), _ptr(logp_ref), _ptr(adv), _ptr(lens), P, G, T, clip_lo, clip_hi, kl_coef,
        agg_mode, _ptr(loss), _ptr(g_logp), _ptr(stats), _ptr(ws), ws.numel() * ws.element_size(), _stream())
    _check(rc, "grpo_loss")


def grpo_loss_noalloc(logp, logp_old, logp_ref, adv, lens, P, G, T, clip_lo, clip_hi, kl_coef, agg_mode,
                      loss, g_logp, stats) -> None:
    rc = load_library().grpo_loss_noalloc(
        _ptr(logp), _ptr(logp_old), _ptr(logp_ref), _ptr(adv), _ptr(lens), P, G, T, clip_lo, clip_hi, kl_coef,
        agg_mode, _ptr(loss), _ptr(g_logp), _ptr(stats), _stream())
    _check(rc, "grpo_loss_noalloc")


def flowrl_tb_loss(logp, logp_ref, reward, logZ, lens, P, G, T, beta, loss, g_logp, g_logZ, resid, ws) -> None:
    rc = load_library().flowrl_tb_loss(
        _ptr(logp), _ptr(logp_ref), _ptr(reward), _ptr(logZ), _ptr(lens), P, G, T, beta, _ptr(loss),
        _ptr(g_logp), _ptr(g_logZ), _ptr(resid), _ptr(ws), ws.numel() * ws.element_size(), _stream())
    _check(rc, "flowrl_tb_loss")


def ce_loss(logp, lens, R, T, loss, g_logp, ws) -> None:
    rc = load_library().ce_loss(_ptr(logp), _ptr(lens), R, T, _ptr(loss), _ptr(g_logp), _ptr(ws),
                                ws.numel() * ws.element_size(), _stream())
    _check(rc, "ce_loss")


def lmhead_check(ws) -> int:
    """Synchronises the current stream; returns 0 or the (negative) sticky device status."""
    return int(load_library().lmhead_check(_ptr(ws), _stream()))


def lmhead_probe_mfma(operands, sink, workgroups: int, iters: int) -> None:
    rc = load_library().lmhead_probe_mfma(_ptr(operands), operands.numel() * operands.element_size(), _ptr(sink),
                                          sink.numel() * sink.element_size(), workgroups, iters, _stream())
    _check(rc, "lmhead_probe_mfma")


def lmhead_timing_enable(on: bool) -> None:
    _check(load_library().lmhead_timing_enable(1 if on else 0), "lmhead_timing_enable")


def lmhead_timing_read(kind: int):
    """(total milliseconds, launches) of one kernel kind since timing was enabled."""
    ms, n = C.c_double(0.0), C.c_int64(0)
    _check(load_library().lmhead_timing_read(kind, C.byref(ms), C.byref(n)), "lmhead_timing_read")
    return ms.value, n.value
