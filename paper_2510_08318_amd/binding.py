"""ctypes binding of liblinattn.so: same names as include/linattn.h, argument marshalling only.

Every step of the operator runs inside the HIP library.  There is no fallback: if the shared
library has not been built, importing a symbol from here raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "liblinattn.so")

OK = 0
E_NULL, E_SHAPE, E_DTYPE, E_ALIGN, E_PHI, E_WORKSPACE, E_HIP, E_STATE, E_ALIAS = range(-1, -10, -1)
PHI_HEDGEHOG = 1
PHI_RELU = 2
BF16, F32, BF16_F32MATH = 1, 2, 3
LAYOUT_BHND, LAYOUT_BNHD = 0, 1
FLAG_CENTRED = 1

EXPORTS = ("linattn_phi_create", "linattn_phi_destroy", "linattn_workspace_bytes", "linattn_workspace_bytes_wgrads",
           "linattn_fwd", "linattn_fwd_noalloc", "linattn_bwd", "linattn_strerror", "linattn_set_stage_events", "linattn_phi_set_blend")


class PhiDesc(ctypes.Structure):
    _fields_ = [
        ("kind", ctypes.c_int), ("dtype", ctypes.c_int), ("H", ctypes.c_int), ("d", ctypes.c_int),
        ("wq", ctypes.c_void_p), ("wk", ctypes.c_void_p),
        ("dwq", ctypes.c_void_p), ("dwk", ctypes.c_void_p),
        ("state", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
        ("layout", ctypes.c_int),
        ("blend_in", ctypes.c_void_p), ("blend_r", ctypes.c_void_p), ("blend_dr", ctypes.c_void_p),
        ("state_bytes", ctypes.c_size_t),
        ("flags", ctypes.c_uint),
    ]


class LinattnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({linattn_strerror(status)})")


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded shared library; fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = ctypes.CDLL(LIB_PATH)
        vp, ci = ctypes.c_void_p, ctypes.c_int
        L.linattn_phi_create.argtypes = [ctypes.POINTER(PhiDesc), ctypes.POINTER(ci)]
        L.linattn_phi_create.restype = ci
        L.linattn_phi_destroy.argtypes = [ci]
        L.linattn_phi_set_blend.argtypes = [ci, vp, vp, vp]
        L.linattn_phi_set_blend.restype = ci
        L.linattn_phi_destroy.restype = ci
        L.linattn_workspace_bytes.argtypes = [ci] * 6
        L.linattn_workspace_bytes.restype = ctypes.c_size_t
        L.linattn_workspace_bytes_wgrads.argtypes = [ci] * 6
        L.linattn_workspace_bytes_wgrads.restype = ctypes.c_size_t
        L.linattn_fwd.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, vp]
        L.linattn_fwd.restype = ci
        L.linattn_fwd_noalloc.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, vp]
        L.linattn_fwd_noalloc.restype = ci
        L.linattn_bwd.argtypes = [vp] * 7 + [ci] * 5 + [vp]
        L.linattn_bwd.restype = ci
        L.linattn_set_stage_events.argtypes = [ctypes.POINTER(vp)]
        L.linattn_set_stage_events.restype = ci
        L.linattn_strerror.argtypes = [ci]
        L.linattn_strerror.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _ptr(x) -> Optional[int]:
    """Device address of a torch tensor, or an integer address passed through (None/0 -> NULL)."""
    if x is None:
        return None
    if isinstance(x, int):
        return x or None
    return int(x.data_ptr()) or None


def linattn_strerror(status: int) -> str:
    return lib().linattn_strerror(int(status)).decode()


def linattn_workspace_bytes(B: int, H: int, n: int, d: int, kind: int = PHI_HEDGEHOG, dtype: int = BF16) -> int:
    return int(lib().linattn_workspace_bytes(B, H, n, d, kind, dtype))


def linattn_workspace_bytes_wgrads(B: int, H: int, n: int, d: int, kind: int = PHI_HEDGEHOG, dtype: int = BF16) -> int:
    return int(lib().linattn_workspace_bytes_wgrads(B, H, n, d, kind, dtype))


def linattn_phi_create(kind, dtype, H, d, wq, wk, dwq=None, dwk=None, state=None,
                       workspace=None, workspace_bytes: int = 0, layout: int = 0,
                       blend_in=None, blend_r=None, blend_dr=None, state_bytes: Optional[int] = None,
                       *, flags: int = 0, check: bool = True) -> int:
    """state_bytes defaults to the size of `state` when that is a tensor."""
    if state_bytes is None:
        state_bytes = 0 if state is None or isinstance(state, int) else state.numel() * state.element_size()
    desc = PhiDesc(int(kind), int(dtype), int(H), int(d), _ptr(wq), _ptr(wk), _ptr(dwq), _ptr(dwk),
                   _ptr(state), _ptr(workspace), int(workspace_bytes), int(layout),
                   _ptr(blend_in), _ptr(blend_r), _ptr(blend_dr), int(state_bytes), int(flags))
    out = ctypes.c_int(-1)
    st = lib().linattn_phi_create(ctypes.byref(desc), ctypes.byref(out))
    if st != OK:
        if check:
            raise LinattnError(st, "linattn_phi_create")
        return st
    return out.value


def linattn_phi_set_blend(phi_id: int, blend_in=None, blend_r=None, blend_dr=None, *, check: bool = True) -> int:
    st = lib().linattn_phi_set_blend(int(phi_id), _ptr(blend_in), _ptr(blend_r), _ptr(blend_dr))
    if st != OK and check:
        raise LinattnError(st, "linattn_phi_set_blend")
    return st


def linattn_phi_destroy(phi_id: int, *, check: bool = True) -> int:
    st = lib().linattn_phi_destroy(int(phi_id))
    if st != OK and check:
        raise LinattnError(st, "linattn_phi_destroy")
    return st


def linattn_fwd(q, k, v, out, B, H, n, d, phi_id, stream=None, *, check: bool = True) -> int:
    st = lib().linattn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(out), B, H, n, d, phi_id, _ptr(stream))
    if st != OK and check:
        raise LinattnError(st, "linattn_fwd")
    return st


def linattn_fwd_noalloc(q, k, v, out, B, H, n, d, phi_id, stream=None, *, check: bool = True) -> int:
    st = lib().linattn_fwd_noalloc(_ptr(q), _ptr(k), _ptr(v), _ptr(out), B, H, n, d, phi_id, _ptr(stream))
    if st != OK and check:
        raise LinattnError(st, "linattn_fwd_noalloc")
    return st


def linattn_bwd(q, k, v, dout, dq, dk, dv, B, H, n, d, phi_id, stream=None, *, check: bool = True) -> int:
    st = lib().linattn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(dout), _ptr(dq), _ptr(dk), _ptr(dv),
                           B, H, n, d, phi_id, _ptr(stream))
    if st != OK and check:
        raise LinattnError(st, "linattn_bwd")
    return st


def linattn_set_stage_events(events) -> int:
    """events: sequence of four hipEvent_t handles (ints), or None to switch instrumentation off."""
    if events is None:
        return lib().linattn_set_stage_events(None)
    arr = (ctypes.c_void_p * 4)(*[int(e) for e in events])
    return lib().linattn_set_stage_events(arr)
