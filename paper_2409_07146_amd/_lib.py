"""ctypes loader for libgsa.so.  There is no fallback: a missing library is an error."""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgsa.so")

# every symbol include/gsa.h declares
EXPORTS = ("gsa_status_string", "gsa_abi_version", "gsa_workspace_bytes", "gsa_fwd", "gsa_bwd", "gsa_fwd_ex", "gsa_bwd_ex",
           "gsa_decode_step", "gsa_decode_workspace_bytes", "gsa_decode_step_ws", "gsa_decode_step_ex",
           "gsa_decode_step_static", "gsa_fwd_act", "gsa_act_slice_cols", "gsa_profile_enable", "gsa_profile_reset", "gsa_profile_read", "gsa_profile_copy")


class GsaProblem(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("T", ctypes.c_int32), ("H", ctypes.c_int32),
                ("d_k", ctypes.c_int32), ("d_v", ctypes.c_int32), ("m", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("scale", ctypes.c_float),
                ("cu_seqlens", ctypes.c_void_p), ("n_seqs", ctypes.c_int32), ("keep_states", ctypes.c_int32)]


_lib = None


def load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            "libgsa.so is not built (%s). Build it with `python -m paper_2409_07146_amd.build` "
            "or __graft_entry__.build(); there is no CPU fallback." % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float
    lib.gsa_status_string.restype = ctypes.c_char_p
    lib.gsa_status_string.argtypes = [ctypes.c_int]
    lib.gsa_abi_version.restype = i32
    lib.gsa_abi_version.argtypes = []
    lib.gsa_workspace_bytes.restype = ctypes.c_int
    lib.gsa_workspace_bytes.argtypes = [ctypes.POINTER(GsaProblem), ctypes.c_int,
                                        ctypes.POINTER(ctypes.c_size_t)]
    lib.gsa_fwd.restype = ctypes.c_int
    lib.gsa_fwd.argtypes = [ctypes.POINTER(GsaProblem)] + [vp] * 10 + [vp, ctypes.c_size_t, vp]
    lib.gsa_bwd.restype = ctypes.c_int
    lib.gsa_bwd.argtypes = [ctypes.POINTER(GsaProblem)] + [vp] * 16 + [vp, ctypes.c_size_t, vp]
    lib.gsa_fwd_ex.restype = ctypes.c_int
    lib.gsa_fwd_ex.argtypes = [ctypes.POINTER(GsaProblem), i32, f32, i32] + [vp] * 11 + [vp, ctypes.c_size_t, vp]
    lib.gsa_fwd_act.restype = ctypes.c_int
    lib.gsa_fwd_act.argtypes = [ctypes.POINTER(GsaProblem), i32, f32, i32] + [vp] * 13 + [vp, ctypes.c_size_t, vp]
    lib.gsa_act_slice_cols.restype = i32
    lib.gsa_act_slice_cols.argtypes = [i32]
    lib.gsa_bwd_ex.restype = ctypes.c_int
    lib.gsa_bwd_ex.argtypes = [ctypes.POINTER(GsaProblem), i32, f32, i32] + [vp] * 18 + [vp, ctypes.c_size_t, vp]
    lib.gsa_decode_step.restype = ctypes.c_int
    lib.gsa_decode_step.argtypes = [i32, i32, i32, i32, i32, i32, f32] + [vp] * 8
    lib.gsa_decode_step_static.restype = ctypes.c_int
    lib.gsa_decode_step_static.argtypes = [i32, i32, i32, i32, i32, i32, f32] + [vp] * 8
    lib.gsa_decode_workspace_bytes.restype = ctypes.c_int
    lib.gsa_decode_workspace_bytes.argtypes = [i32, i32, i32, i32, i32, ctypes.POINTER(ctypes.c_size_t)]
    lib.gsa_decode_step_ws.restype = ctypes.c_int
    lib.gsa_decode_step_ws.argtypes = [i32, i32, i32, i32, i32, i32, f32] + [vp] * 7 + [vp, ctypes.c_size_t, vp]
    lib.gsa_decode_step_ex.restype = ctypes.c_int
    lib.gsa_decode_step_ex.argtypes = [i32, i32, i32, i32, i32, i32, f32, i32, f32, i32] + [vp] * 8 + [vp, ctypes.c_size_t, vp]
    lib.gsa_profile_enable.restype = ctypes.c_int
    lib.gsa_profile_enable.argtypes = [ctypes.c_int]
    lib.gsa_profile_reset.restype = ctypes.c_int
    lib.gsa_profile_reset.argtypes = []
    lib.gsa_profile_read.restype = ctypes.c_int
    lib.gsa_profile_read.argtypes = [i32, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(ctypes.c_double),
                                     ctypes.POINTER(ctypes.c_int64)]
    lib.gsa_profile_copy.restype = ctypes.c_int
    lib.gsa_profile_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
    _lib = lib
    return lib
