"""ctypes binding of the KV-compression entry points of liblmhead.so (``include/dynakv.h``):
argument marshalling only.  Same conventions as ``binding.py``: torch CUDA (ROCm) tensors in, the
current stream, ``LmheadError`` on a negative status.  Nothing is computed here.
"""
from __future__ import annotations

import ctypes as C

from .binding import LMHEAD_BF16, LMHEAD_F32, _check, _ptr, _stream, load_library

DYNAKV_SYMBOLS = [
    "dynakv_workspace_bytes", "dynakv_validate_desc", "dynakv_gate", "dynakv_store",
    "dynakv_reconstruct", "dynakv_retain", "dynakv_check", "dynakv_bwd_workspace_bytes", "dynakv_gate_bwd",
]

FLAG_LITERAL_FLIP = 1 << 0
FLAG_ACCUM_GRAD = 1 << 1
GRANULE = 8


class DynakvDesc(C.Structure):
    _fields_ = [
        ("n", C.c_int32), ("d", C.c_int32), ("dtype", C.c_int32), ("flags", C.c_uint32),
        ("ldx", C.c_int64), ("reserved", C.c_int64),
    ]


_ready = False


def _lib():
    global _ready
    lib = load_library()
    if not _ready:
        vp, i64, f32, sz = C.c_void_p, C.c_int64, C.c_float, C.c_size_t
        dp = C.POINTER(DynakvDesc)
        lib.dynakv_workspace_bytes.restype = sz
        lib.dynakv_workspace_bytes.argtypes = [dp]
        lib.dynakv_validate_desc.restype = C.c_int
        lib.dynakv_validate_desc.argtypes = [dp]
        lib.dynakv_gate.restype = C.c_int
        lib.dynakv_gate.argtypes = [dp, vp, vp, vp, vp, f32, vp, vp, vp, vp, vp, sz, vp]
        lib.dynakv_store.restype = C.c_int
        lib.dynakv_store.argtypes = [dp, vp, vp, i64, vp, vp, i64, vp, sz, vp]
        lib.dynakv_reconstruct.restype = C.c_int
        lib.dynakv_reconstruct.argtypes = [dp, vp, i64, vp, vp, vp, vp, vp, sz, vp]
        lib.dynakv_retain.restype = C.c_int
        lib.dynakv_retain.argtypes = [dp, vp, vp, f32, vp, vp, vp, sz, vp]
        lib.dynakv_bwd_workspace_bytes.restype = sz
        lib.dynakv_bwd_workspace_bytes.argtypes = [dp]
        lib.dynakv_gate_bwd.restype = C.c_int
        lib.dynakv_gate_bwd.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, f32, vp, vp, vp, vp, vp, sz, vp]
        lib.dynakv_check.restype = C.c_int
        lib.dynakv_check.argtypes = [vp, vp]
        _ready = True
    return lib


def make_kv_desc(n, d, dtype, ldx=None, flags=0) -> DynakvDesc:
    code = {"bf16": LMHEAD_BF16, "f32": LMHEAD_F32}.get(dtype, dtype)
    return DynakvDesc(n=n, d=d, dtype=code, flags=flags, ldx=d if ldx is None else ldx, reserved=0)


def dynakv_workspace_bytes(desc: DynakvDesc) -> int:
    return int(_lib().dynakv_workspace_bytes(C.byref(desc)))


def dynakv_validate_desc(desc: DynakvDesc) -> int:
    return int(_lib().dynakv_validate_desc(C.byref(desc)))


def _nbytes(t) -> int:
    return t.numel() * t.element_size()


def dynakv_gate(desc, x, U, W, b, tau, xt, k, m, xhat, ws) -> None:
    rc = _lib().dynakv_gate(C.byref(desc), _ptr(x), _ptr(U), _ptr(W), _ptr(b), tau, _ptr(xt), _ptr(k), _ptr(m),
                            _ptr(xhat), _ptr(ws), _nbytes(ws), _stream())
    _check(rc, "dynakv_gate")


def dynakv_store(desc, xt, k, off_base, off, packed, capacity, ws) -> None:
    rc = _lib().dynakv_store(C.byref(desc), _ptr(xt), _ptr(k), off_base, _ptr(off), _ptr(packed), capacity,
                             _ptr(ws), _nbytes(ws), _stream())
    _check(rc, "dynakv_store")


def dynakv_reconstruct(desc, packed, packed_elems, off, k, U_inv, xbar, ws) -> None:
    rc = _lib().dynakv_reconstruct(C.byref(desc), _ptr(packed), packed_elems, _ptr(off), _ptr(k), _ptr(U_inv),
                                   _ptr(xbar), _ptr(ws), _nbytes(ws), _stream())
    _check(rc, "dynakv_reconstruct")


def dynakv_retain(desc, k, m, alpha, out, g_m, ws) -> None:
    rc = _lib().dynakv_retain(C.byref(desc), _ptr(k), _ptr(m), alpha, _ptr(out), _ptr(g_m), _ptr(ws), _nbytes(ws),
                              _stream())
    _check(rc, "dynakv_retain")


def dynakv_bwd_workspace_bytes(desc: DynakvDesc) -> int:
    return int(_lib().dynakv_bwd_workspace_bytes(C.byref(desc)))


def dynakv_gate_bwd(desc, x, U, W, b, xt, g_xhat, g_m, g_m_const, dx, dU, dW, db, ws) -> None:
    rc = _lib().dynakv_gate_bwd(C.byref(desc), _ptr(x), _ptr(U), _ptr(W), _ptr(b), _ptr(xt), _ptr(g_xhat),
                                _ptr(g_m), g_m_const, _ptr(dx), _ptr(dU), _ptr(dW), _ptr(db), _ptr(ws),
                                _nbytes(ws), _stream())
    _check(rc, "dynakv_gate_bwd")


def dynakv_check(ws) -> int:
    """Synchronises the current stream; returns 0 or the (negative) device status of the last call."""
    return int(_lib().dynakv_check(_ptr(ws), _stream()))
