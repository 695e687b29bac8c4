"""Loads libqn.so (built in-tree by paper_1709_05069_amd/build.py)."""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libqn.so")

_i64 = ctypes.c_int64
_int = ctypes.c_int
_f32 = ctypes.c_float
_vp = ctypes.c_void_p

_sz = ctypes.c_size_t

# name -> (restype, argtypes); mirrors include/qn.h and include/qn_diag.h
SIGNATURES = {
    "qn_workspace_bytes": (_sz, [_i64, _int, _int]),
    "qn_update_ws": (_int, [_vp, _vp, _int, _i64, _int, _i64, _f32, _f32, _vp, _vp,
                            _vp, _sz, _vp]),
    "qn_update_noalloc": (_int, [_vp, _vp, _int, _i64, _int, _i64, _f32, _f32, _vp, _vp,
                                 _vp]),
    "qn_gram_state_bytes": (_sz, []),
    "qn_gram_state_init_ws": (_int, [_vp, _int, _i64, _int, _i64, _vp, _vp, _sz, _vp]),
    "qn_gram_state_write_ws": (_int, [_vp, _int, _i64, _int, _i64, _int, _vp, _vp, _sz, _vp]),
    "qn_gram_state_get": (_int, [_vp, _int, _vp, _vp, _vp]),
    "qn_update_async_ws": (_int, [_vp, _vp, _int, _i64, _int, _i64, _int, _f32, _f32, _vp,
                                  _vp, _vp, _vp, _sz, _vp]),
    "qn_gram_ws": (_int, [_vp, _int, _i64, _int, _i64, _vp, _vp, _vp, _sz, _vp]),
    "qn_hinv_ws": (_int, [_vp, _vp, _int, _vp, _i64, _int, _i64, _f32, _vp, _vp,
                          _vp, _sz, _vp]),
    "qn_gemv_t_ws": (_int, [_vp, _int, _vp, _i64, _int, _i64, _vp, _vp, _sz, _vp]),
    "qn_update_bounded_ws": (_int, [_vp, _vp, _int, _i64, _int, _i64, _f32, _f32, _int,
                                    _vp, _vp, _vp, _vp, _sz, _vp]),
    "qn_diag_gram_ex": (_int, [_vp, _int, _vp, _i64, _int, _i64, _int, _vp, _vp, _vp]),
    "qn_status_string": (ctypes.c_char_p, [_int]),
    "qn_kernel_name": (ctypes.c_char_p, [_int]),
    "qn_init": (_int, []),
    "qn_shutdown": (_int, []),
    "qn_update": (_int, [_vp, _vp, _i64, _int, _f32, _f32, _vp, _vp, _vp]),
    "qn_update_bf16": (_int, [_vp, _vp, _i64, _int, _f32, _f32, _vp, _vp, _vp]),
    "qn_gram": (_int, [_vp, _i64, _int, _vp, _vp, _vp]),
    "qn_gram_bf16": (_int, [_vp, _i64, _int, _vp, _vp, _vp]),
    "qn_eig": (_int, [_vp, _vp, _int, _f32, _vp, _vp, _vp, _vp, _vp]),
    "qn_apply": (_int, [_vp, _vp, _i64, _int, _vp, _f32, _vp, _vp]),
    "qn_apply_bf16": (_int, [_vp, _vp, _i64, _int, _vp, _f32, _vp, _vp]),
    "qn_update_ex": (_int, [_vp, _vp, _int, _i64, _int, _i64, _f32, _f32, _vp,
                            _vp, _vp]),
    "qn_gram_ex": (_int, [_vp, _int, _i64, _int, _i64, _vp, _vp, _vp]),
    "qn_apply_ex": (_int, [_vp, _vp, _int, _i64, _int, _i64, _vp, _f32, _vp,
                           _vp]),
    "qn_hinv": (_int, [_vp, _vp, _vp, _i64, _int, _f32, _vp, _vp, _vp]),
    "qn_hinv_bf16": (_int, [_vp, _vp, _vp, _i64, _int, _f32, _vp, _vp, _vp]),
    "qn_hinv_ex": (_int, [_vp, _vp, _int, _vp, _i64, _int, _i64, _f32, _vp, _vp,
                          _vp]),
    "qn_gemv_t_ex": (_int, [_vp, _int, _vp, _i64, _int, _i64, _vp, _vp]),
    "qn_coef": (_int, [_vp, _vp, _vp, _vp, _int, _vp, _vp]),
    "qn_hinv_apply_ex": (_int, [_vp, _vp, _int, _vp, _i64, _int, _i64, _vp, _vp,
                                _vp]),
    "qn_update_bounded_ex": (_int, [_vp, _vp, _int, _i64, _int, _i64, _f32, _f32, _int,
                                    _vp, _vp, _vp, _vp]),
    "qn_tau_bound": (_int, [_vp, _vp, _vp, _vp, _int, _f32, _int, _vp, _vp, _vp]),
    "qn_probe_copy": (_int, [_vp, _vp, _i64, _vp]),
    "qn_probe_read": (_int, [_vp, _i64, _vp, _vp]),
    "qn_probe_chain": (_int, [_i64, _vp, _vp]),
    "qn_probe_sink_floats": (_int, []),
    "qn_trace_begin": (_int, [_int]),
    "qn_trace_end": (_int, [_vp, _vp]),
}

_LIB = None


def load():
    """Returns the ctypes handle; raises if the library has not been built."""
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it first "
                "(python -m paper_1709_05069_amd.build). "
                "There is no fallback path.")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)   # AttributeError if a symbol is missing
            fn.restype = res
            fn.argtypes = args
        _LIB = lib
    return _LIB
