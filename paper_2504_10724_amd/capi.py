"""Thin ctypes binding of libee: the same names as include/ee.h, argument
marshalling only.  Every step of the decode path runs in the library's HIP
kernels; there is no fallback: if the shared library is missing, importing a
symbol from it raises."""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("EE_LIB_PATH", os.path.join(HERE, "libee.so"))

EE_MAX_EXITS = 16
EE_OK = 0
EE_ERR_INVALID_ARG, EE_ERR_SHAPE, EE_ERR_CAPACITY = -1, -2, -3
EE_ERR_LAYER_NOT_RESIDENT, EE_ERR_EXIT_NOT_RESIDENT, EE_ERR_DTYPE, EE_ERR_HIP = -4, -5, -6, -7
EE_F32, EE_BF16 = 0, 1


class ee_model_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32),
                ("vocab", C.c_int32), ("dtype", C.c_int32), ("rms_eps", C.c_float),
                ("rope_theta", C.c_float), ("max_pos", C.c_int32), ("n_exits", C.c_int32),
                ("exit_layers", C.c_int32 * EE_MAX_EXITS)]


class ee_layer_weights(C.Structure):
    _fields_ = [("g_attn", C.c_void_p), ("w_qkv", C.c_void_p), ("w_o", C.c_void_p),
                ("g_ffn", C.c_void_p), ("w_gate_up", C.c_void_p), ("w_down", C.c_void_p)]


class ee_batch_layout(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in (
        "h", "tok_in", "pos", "row_scale", "active_idx", "n_active", "exited_idx", "n_exited",
        "head_conf", "head_tok", "head_exit", "head_breach", "out_tok", "out_layer", "out_conf",
        "out_breach", "exit_counts", "breach_count", "status")]


class ee_pht_row(C.Structure):
    _fields_ = [("tokens", C.c_int64), ("breaches", C.c_int64), ("exits", C.c_int64 * EE_MAX_EXITS),
                ("nll", C.c_double)]


_vp, _i, _sz, _f = C.c_void_p, C.c_int, C.c_size_t, C.c_float
_SIGS = {
    "ee_last_error": (C.c_char_p, []),
    "ee_device_count": (_i, []),
    "ee_packed_bytes": (_sz, [_i, _i]),
    "ee_pack_weight": (_i, [_vp, _i, _i, _vp, _i, _i, _i, _vp]),
    "ee_model_create": (_i, [C.POINTER(ee_model_config), C.POINTER(_vp)]),
    "ee_model_destroy": (_i, [_vp]),
    "ee_model_set_layer": (_i, [_vp, _i, C.POINTER(ee_layer_weights)]),
    "ee_model_set_exit": (_i, [_vp, _i, _vp, _vp]),
    "ee_model_set_embed": (_i, [_vp, _vp]),
    "ee_model_resident_depth": (_i, [_vp]),
    "ee_kv_pool_bytes": (_sz, [_vp, _i, C.POINTER(C.c_int32), _i]),
    "ee_kv_bind": (_i, [_vp, _vp, _sz, _i, C.POINTER(C.c_int32), _i, C.POINTER(_vp)]),
    "ee_kv_destroy": (_i, [_vp]),
    "ee_kv_write_context": (_i, [_vp, _vp, _i, _i, _i, _i, _vp, _vp, _vp]),
    "ee_kv_read_context": (_i, [_vp, _vp, _i, _i, _i, _i, _vp, _vp, _vp]),
    "ee_batch_state_bytes": (_sz, [_vp, _i]),
    "ee_workspace_bytes": (_sz, [_vp, _i]),
    "ee_batch_bind": (_i, [_vp, _i, _vp, _sz, _vp, _sz, C.POINTER(_vp)]),
    "ee_batch_destroy": (_i, [_vp]),
    "ee_batch_get_layout": (_i, [_vp, _i, C.POINTER(ee_batch_layout)]),
    "ee_batch_reset": (_i, [_vp, _vp, _vp, _vp, _vp]),
    "ee_batch_set_row_scale": (_i, [_vp, _vp, _vp]),
    "ee_batch_begin_step": (_i, [_vp, _vp, _vp]),
    "ee_layer_forward": (_i, [_vp, _i, _vp, _vp, _vp]),
    "ee_exit_head": (_i, [_vp, _i, _f, _i, _vp, _vp, _vp]),
    "ee_exit_head_static": (_i, [_vp, _i, _f, _i, _vp, _vp]),
    "ee_compact_active": (_i, [_vp, _i, _i, _vp]),
    "ee_fill_skipped_kv": (_i, [_vp, _i, _i, _vp, _vp, _vp]),
    "ee_decode_step": (_i, [_vp, _vp, _vp, C.POINTER(C.c_float), _i, _vp]),
    "ee_decode_segment": (_i, [_vp, _vp, _vp, C.POINTER(C.c_float), _i, _i, _vp]),
    "ee_decode_finish": (_i, [_vp, _vp, _vp, _i, _vp]),
    "ee_prefill": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _i, _vp]),
    "ee_draft_step": (_i, [_vp, _vp, _vp, _i, _vp, _vp]),
    "ee_verify_drafts": (_i, [_vp, _vp, _vp, _vp, _i, _i, _vp, _vp, _vp, _vp, _vp]),
    "ee_model_set_layer_on": (_i, [_vp, _i, C.POINTER(ee_layer_weights), _vp]),
    "ee_hstore_bytes": (_sz, [_vp, _vp]),
    "ee_hstore_put_step": (_i, [_vp, _vp, _vp, _vp, _vp]),
    "ee_hstore_put_prefill": (_i, [_vp, _vp, _vp, _i, _vp, _vp]),
    "ee_backfill_kv": (_i, [_vp, _i, _i, _vp, _vp, _vp, _vp, _vp, _i, _vp]),
    "ee_cbc_state_bytes": (C.c_size_t, [_i]),
    "ee_cbc_init": (_i, [_vp, _i, _i, _vp]),
    "ee_cbc_push": (_i, [_vp, _vp, _i, _vp]),
    "ee_cbc_push_step": (_i, [_vp, _vp, _vp]),
    "ee_pht_init": (_i, [_vp, _vp]),
    "ee_pht_push_step": (_i, [_vp, _vp, _vp, _vp]),
    "ee_timing_enable": (_i, [_i]),
    "ee_timing_reset": (_i, []),
    "ee_timing_read": (_i, [_i, C.POINTER(_i), C.POINTER(_f)]),
}
KERNEL_CLASSES = ["embed", "norm", "gemm_qkv", "rope_append", "attention", "gemm_o", "gemm_gate_up", "gemm_down",
                  "exit_gemm", "exit_decide", "compact", "fill_kv", "cbc", "pht"]

_lib = None


def load():
    """Loads paper_2504_10724_amd/libee.so (built by build.py).  Raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built: run `python -m paper_2504_10724_amd.build` "
                              "(there is no fallback path)")
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGS.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def exported_names():
    return list(_SIGS)


class EEError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libee error {code}: {msg}")
        self.code = code


def check(rc):
    if rc != EE_OK:
        raise EEError(rc, load().ee_last_error().decode())
    return rc


def __getattr__(name):
    if name in _SIGS:
        return getattr(load(), name)
    raise AttributeError(name)
