"""ctypes loader for libloract.so.  Fails loudly when the library has not been built."""
from __future__ import annotations

import ctypes
import os

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG_DIR, "libloract.so")


class LoractParams(ctypes.Structure):
    """Mirror of `loract_params` in include/loract.h."""
    _fields_ = [
        ("m", ctypes.c_int64),
        ("n", ctypes.c_int64),
        ("ldx", ctypes.c_int64),
        ("k", ctypes.c_int32),
        ("l", ctypes.c_int32),
        ("t", ctypes.c_int32),
        ("x_dtype", ctypes.c_int32),
        ("factor_dtype", ctypes.c_int32),
        ("seed", ctypes.c_uint64),
    ]


_P = ctypes.POINTER
_vp, _i32, _i64, _u64, _sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64, ctypes.c_size_t

# name -> (restype, argtypes); one entry per symbol declared in include/loract.h
SIGNATURES = {
    "loract_version": (ctypes.c_char_p, []),
    "loract_strerror": (ctypes.c_char_p, [ctypes.c_int]),
    "loract_last_hip_error": (ctypes.c_char_p, []),
    "loract_sample_indices": (ctypes.c_int, [_i64, _i32, _u64, _P(_i32)]),
    "loract_workspace_bytes": (ctypes.c_int, [_P(LoractParams), _P(_sz)]),
    "loract_compress": (ctypes.c_int, [_vp, _P(LoractParams), _P(_i32), _vp, _vp, _vp, _sz, _vp, _vp]),
    "loract_compress_adaptive": (ctypes.c_int, [_vp, _P(LoractParams), _P(_i32), ctypes.c_double, _vp, _vp, _vp,
                                                _vp, _sz, _vp, _vp]),
    "loract_reconstruct": (ctypes.c_int, [_vp, _vp, _i64, _i64, _i32, _i32, _vp, _i64, _i32, _vp]),
    "loract_lora_grad_workspace_bytes": (ctypes.c_int, [_i64, _i64, _i32, _i64, _i32, _P(_sz)]),
    "loract_lora_grad": (ctypes.c_int, [_vp, _vp, _i64, _i64, _i32, _i32, _vp, _i64, _vp, _i32, _i32,
                                        ctypes.c_float, _vp, _vp, _sz, _vp]),
    "loract_static_scratch_bytes": (_sz, []),
    "loract_lora_grad_static": (ctypes.c_int, [_vp, _vp, _i64, _i64, _i32, _i32, _vp, _i64, _vp, _i32, _i32,
                                               ctypes.c_float, _vp, _vp]),
    "loract_rsvd": (ctypes.c_int, [_vp, _P(LoractParams), _vp, _vp, _vp, _vp, _sz, _vp, _vp]),
    "loract_gaussian_omega_t": (ctypes.c_int, [_vp, _i32, _i64, _i32, _u64, _vp]),
    "loract_prenorm_forward": (ctypes.c_int, [_vp, _i64, _i64, _i64, _i32, _vp, ctypes.c_float, _vp, _i64,
                                              _vp, _vp]),
    "loract_prenorm_backward": (ctypes.c_int, [_vp, _i64, _i64, _i64, _i32, _vp, _vp, _vp, _i64, _vp,
                                               _i64, _vp]),
    "loract_profile_begin": (ctypes.c_int, []),
    "loract_profile_end": (ctypes.c_int, []),
    "loract_profile_count": (ctypes.c_int, []),
    "loract_profile_get": (ctypes.c_int, [ctypes.c_int, ctypes.c_char_p, ctypes.c_int,
                                          _P(ctypes.c_double), _P(_i64)]),
}

_lib = None


def load() -> ctypes.CDLL:
    """Load the shared library once and attach the C signatures."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            "libloract.so is missing (%s). Build it with `python -m paper_2509_23472_amd.build` "
            "or __graft_entry__.build(); there is no CPU fallback." % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    for name, (restype, argtypes) in SIGNATURES.items():
        fn = getattr(lib, name)          # AttributeError if the symbol is not exported
        fn.restype = restype
        fn.argtypes = argtypes
    _lib = lib
    return lib
