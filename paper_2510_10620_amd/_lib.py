"""ctypes loader for libdcp_attn.so.  There is no fallback: if the library is missing it is
built once with hipcc; if that fails the import error propagates."""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("DCP_LIB_PATH") or os.path.join(HERE, "libdcp_attn.so")   # DCP_LIB_PATH: load another build of the same library

i32p = ctypes.POINTER(ctypes.c_int32)
i64p = ctypes.POINTER(ctypes.c_int64)
vp = ctypes.c_void_p


class Tensors(ctypes.Structure):
    """Mirror of dcp_tensors_t (include/dcp.h)."""
    _fields_ = [
        ("hq", ctypes.c_int32), ("hkv", ctypes.c_int32), ("d", ctypes.c_int32),
        ("dtype", ctypes.c_int32), ("impl", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
        ("q", vp), ("q_stride_t", ctypes.c_int64), ("q_stride_h", ctypes.c_int64),
        ("k", vp), ("k_stride_t", ctypes.c_int64), ("k_stride_h", ctypes.c_int64),
        ("v", vp), ("v_stride_t", ctypes.c_int64), ("v_stride_h", ctypes.c_int64),
        ("attn_ranges", vp),
        ("out", vp), ("o_stride_t", ctypes.c_int64), ("o_stride_h", ctypes.c_int64),
        ("lse", vp),
        ("dout", vp), ("do_stride_t", ctypes.c_int64), ("do_stride_h", ctypes.c_int64),
        ("dq", vp), ("dq_stride_t", ctypes.c_int64), ("dq_stride_h", ctypes.c_int64),
        ("dk", vp), ("dk_stride_t", ctypes.c_int64), ("dk_stride_h", ctypes.c_int64),
        ("dv", vp), ("dv_stride_t", ctypes.c_int64), ("dv_stride_h", ctypes.c_int64),
    ]


class Instr(ctypes.Structure):
    """dcp_instr_t"""
    _fields_ = [
        ("op", ctypes.c_int32), ("comm_id", ctypes.c_int32),
        ("plan", vp),
        ("tensors", Tensors),
        ("workspace", vp), ("workspace_bytes", ctypes.c_size_t),
        ("o_part", vp), ("lse_part", vp),
        ("copy_list", vp),
        ("src", vp), ("dst", vp),
        ("src_row_stride", ctypes.c_int64), ("dst_row_stride", ctypes.c_int64), ("row_bytes", ctypes.c_int64),
        ("parts", vp * 8),
        ("n_parts", ctypes.c_int32), ("parts_dtype", ctypes.c_int32), ("dst_dtype", ctypes.c_int32),
        ("n_elems", ctypes.c_int64),
    ]


_SIGS = {
    "dcp_build_block_table": (ctypes.c_int, [i32p, ctypes.c_int32, ctypes.c_int32, i32p, i32p, ctypes.c_int64, i64p]),
    "dcp_count_pairs": (ctypes.c_int, [i32p, ctypes.c_int32, ctypes.c_int32, i32p, ctypes.c_int64, i32p, i64p]),
    "dcp_build_block_table_window": (ctypes.c_int, [i32p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, i32p,
                                                    ctypes.c_int64, i64p]),
    "dcp_count_pairs_window": (ctypes.c_int, [i32p, ctypes.c_int32, ctypes.c_int32, i32p, ctypes.c_int64, ctypes.c_int32,
                                              ctypes.c_int32, i64p]),
    "dcp_plan_set_window": (ctypes.c_int, [vp, ctypes.c_int32, ctypes.c_int32]),
    "dcp_program_create": (ctypes.c_int, [ctypes.POINTER(vp), ctypes.POINTER(Instr), ctypes.c_int64]),
    "dcp_program_destroy": (ctypes.c_int, [vp]),
    "dcp_program_run": (ctypes.c_int, [vp, vp, vp]),
    "dcp_comm_volume": (ctypes.c_int, [i32p, ctypes.c_int32, ctypes.c_int32, i32p, ctypes.c_int64, i32p, i32p, ctypes.c_int32,
                                       ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, i64p, i64p, i64p, i64p, i64p]),
    "dcp_plan_create": (ctypes.c_int, [ctypes.POINTER(vp), i32p, ctypes.c_int32, ctypes.c_int32, i32p, ctypes.c_int64, i32p, ctypes.c_int32]),
    "dcp_plan_set_block_buffers": (ctypes.c_int, [vp, i32p, ctypes.c_int32, i32p, ctypes.c_int32]),
    "dcp_plan_destroy": (ctypes.c_int, [vp]),
    "dcp_plan_prepare": (ctypes.c_int, [vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp]),
    "dcp_plan_export": (ctypes.c_int, [vp, ctypes.c_int, i32p, ctypes.c_int64, i64p]),
    "dcp_plan_export_dkv_items": (ctypes.c_int, [vp, ctypes.c_int32, i32p, ctypes.c_int64, i64p]),
    "dcp_plan_export_dkv_segments": (ctypes.c_int, [vp, ctypes.c_int32, i32p, i32p]),
    "dcp_block_attn_fwd": (ctypes.c_int, [vp, ctypes.POINTER(Tensors), vp]),
    "dcp_merge_partials": (ctypes.c_int, [vp, vp, vp, vp, ctypes.c_int64, ctypes.c_int64, vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp]),
    "dcp_bwd_delta": (ctypes.c_int, [ctypes.POINTER(Tensors), ctypes.c_int64, vp, vp]),
    "dcp_bwd_workspace_bytes": (ctypes.c_size_t, [vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]),
    "dcp_block_attn_bwd": (ctypes.c_int, [vp, ctypes.POINTER(Tensors), vp, ctypes.c_size_t, vp]),
    "dcp_block_attn_bwd_static": (ctypes.c_int, [vp, ctypes.POINTER(Tensors), vp]),
    "dcp_sum_partials": (ctypes.c_int, [ctypes.POINTER(vp), ctypes.c_int32, ctypes.c_int32, vp, ctypes.c_int32, ctypes.c_int64, vp]),
    "dcp_copy_list_create": (ctypes.c_int, [ctypes.POINTER(vp), i32p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64]),
    "dcp_copy_list_destroy": (ctypes.c_int, [vp]),
    "dcp_blockwise_copy": (ctypes.c_int, [vp, vp, ctypes.c_int64, vp, ctypes.c_int64, ctypes.c_int64, vp]),
    "dcp_profile_enable": (ctypes.c_int, [ctypes.c_int32]),
    "dcp_profile_read": (ctypes.c_int, [ctypes.c_int32, ctypes.POINTER(ctypes.c_double), i64p]),
    "dcp_last_error": (ctypes.c_char_p, []),
    "dcp_version": (ctypes.c_char_p, []),
}

_lib = None


def load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build(verbose=False)
    # torch first: it brings its own copy of the HIP runtime, and the device tensors this binding is handed live in
    # that copy.  Loaded after torch, the library binds to the same runtime; loaded before it, the process would hold
    # two runtimes and the library's own would find no device ("no ROCm-capable device is detected").
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    for name, (res, args) in _SIGS.items():
        fn = getattr(lib, name)          # AttributeError if the symbol is not exported
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def exported_names():
    return list(_SIGS)
