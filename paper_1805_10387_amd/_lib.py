"""ctypes loader for libmp.so and the C structs of include/mp.h."""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmp.so")   # the in-tree build, and nothing else

MP_HISTORY = 4096
MP_OK, MP_E_INVAL, MP_E_UNSUPPORTED, MP_E_WORKSPACE, MP_E_HIP = 0, -1, -2, -3, -4
MP_SCALE_STATIC, MP_SCALE_BACKOFF = 0, 1
MP_EPI_NONE, MP_EPI_BIAS, MP_EPI_BIAS_RELU = 0, 1, 2
MP_OPT_SGD, MP_OPT_ADAM = 0, 1
MP_UPDATE_DEFAULT, MP_UPDATE_PRECHECKED = 0, 1


class ScaleState(C.Structure):
    _fields_ = [("scale", C.c_float), ("inv_scale", C.c_float), ("min_scale", C.c_float), ("max_scale", C.c_float),
                ("mode", C.c_int32), ("growth_interval", C.c_int32), ("good_steps", C.c_int32), ("found_inf", C.c_int32),
                ("opt_step", C.c_int32), ("total_steps", C.c_int32), ("skipped_steps", C.c_int32), ("reserved", C.c_int32),
                ("hist_scale", C.c_float * MP_HISTORY), ("hist_found_inf", C.c_int32 * MP_HISTORY)]


class GemmDesc(C.Structure):
    _fields_ = [("M", C.c_int32), ("N", C.c_int32), ("K", C.c_int32),
                ("ldx", C.c_int32), ("ldw", C.c_int32), ("ldy", C.c_int32),
                ("batch_outer", C.c_int32), ("batch_inner", C.c_int32),
                ("sx_outer", C.c_int64), ("sx_inner", C.c_int64),
                ("sw_outer", C.c_int64), ("sw_inner", C.c_int64),
                ("sy_outer", C.c_int64), ("sy_inner", C.c_int64),
                ("alpha", C.c_float), ("epilogue", C.c_int32), ("trans_w", C.c_int32), ("reserved", C.c_int32)]


class GemmGroupItem(C.Structure):
    _fields_ = [("desc", GemmDesc), ("dY", C.c_void_p), ("X", C.c_void_p), ("dW", C.c_void_p), ("db", C.c_void_p)]


class LstmLayerDesc(C.Structure):
    _fields_ = [("T", C.c_int32), ("B", C.c_int32), ("I", C.c_int32), ("H", C.c_int32),
                ("ldw", C.c_int32), ("ldxh", C.c_int32), ("ld_up", C.c_int32), ("wait_limit_us", C.c_int32),
                ("debug_extra_participants", C.c_int32), ("reserved", C.c_int32)]


class TensorDesc(C.Structure):
    _fields_ = [("g16", C.c_void_p), ("w32", C.c_void_p), ("w16", C.c_void_p), ("m", C.c_void_p), ("v", C.c_void_p),
                ("n", C.c_size_t)]


class OptCfg(C.Structure):
    _fields_ = [("kind", C.c_int32), ("reserved", C.c_int32), ("lr", C.c_double), ("beta1", C.c_double),
                ("beta2", C.c_double), ("eps", C.c_double), ("weight_decay", C.c_double)]


_P, _I, _I64, _SZ, _F = C.c_void_p, C.c_int, C.c_int64, C.c_size_t, C.c_float

# name -> (restype, argtypes); must list every symbol include/mp.h declares
SIGNATURES = {
    "mp_last_error": (C.c_char_p, []),
    "mp_version": (_I, []),
    "mp_scale_state_init": (_I, [_P, _I, _F, _I, _F, _F, _P]),
    "mp_loss_scale_update": (_I, [_P, _P]),
    "mp_gemm_bwd_dw_workspace_bytes": (_SZ, [C.POINTER(GemmDesc), _I]),
    "mp_gemm_fwd": (_I, [C.POINTER(GemmDesc), _P, _P, _P, _P, _P, _P, _P]),
    "mp_gemm_bwd_dx": (_I, [C.POINTER(GemmDesc), _P, _P, _P, _P, C.c_int32, _P, _P]),
    "mp_gemm_bwd_dw": (_I, [C.POINTER(GemmDesc), _P, _P, _P, _P, _P, _P, _SZ, _P]),
    "mp_gemm_split_workspace_bytes": (_SZ, [C.POINTER(GemmDesc)]),
    "mp_gemm_fwd_ws": (_I, [C.POINTER(GemmDesc), _P, _P, _P, _P, _P, _P, _P, _SZ, _P]),
    "mp_gemm_bwd_dx_ws": (_I, [C.POINTER(GemmDesc), _P, _P, _P, _P, C.c_int32, _P, _P, _SZ, _P]),
    "mp_gemm_bwd_dw_grouped": (_I, [C.POINTER(GemmGroupItem), _I, _P, _P]),
    "mp_gemm_tuning_override": (_I, [_I, _I]),
    "mp_gemm_tuning_dtl": (_I, [_I]),
    "mp_colsum_workspace_bytes": (_SZ, [_I, _I]),
    "mp_colsum": (_I, [_I, _I, _P, _I, _P, _P, _P, _SZ, _P]),
    "mp_colsum_static_max_bytes": (_SZ, []),
    "mp_colsum_static": (_I, [_I, _I, _P, _I, _P, _P, _P]),
    "mp_loss_workspace_bytes": (_SZ, [_I, _I]),
    "mp_mse_scaled": (_I, [_I, _I, _P, _P, _I, _P, _P, _P, _P, _SZ, _P]),
    "mp_softmax_xent_scaled": (_I, [_I, _I, _P, _I, _P, _P, _P, _P, _P, _SZ, _P]),
    "mp_softmax_xent_db_workspace_bytes": (_SZ, [_I, _I]),
    "mp_softmax_xent_scaled_db": (_I, [_I, _I, _P, _I, _P, _P, _P, _P, _P, _P, _SZ, _P]),
    "mp_layernorm_fwd": (_I, [_I, _I, _P, _P, _P, _P, _F, _P, _P, _P, _P]),
    "mp_layernorm_bwd_workspace_bytes": (_SZ, [_I, _I]),
    "mp_layernorm_bwd": (_I, [_I, _I, _P, _P, _P, _P, _P, _P, _P, _P, _P, _P, _P, _P, _SZ, _P]),
    "mp_softmax_fwd": (_I, [_I64, _I, _P, _P, _I, _P]),
    "mp_softmax_bwd": (_I, [_I64, _I, _P, _P, _P, _I, _P]),
    "mp_attention_fwd": (_I, [_I, _I, _I, _I, _P, _I, _F, _P, _P, _I, _P]),
    "mp_attention_bwd": (_I, [_I, _I, _I, _I, _P, _I, _F, _P, _P, _I, _P, _I, _P]),
    "mp_lstm_cell_fwd": (_I, [_I, _I, _P, _I, _P, _P, _P, _I, _P, _I, _P]),
    "mp_lstm_cell_bwd": (_I, [_I, _I, _P, _I, _P, _P, _P, _I, _P, _I, _P, _P, _P]),
    "mp_lstm_layer_workspace_bytes": (_SZ, []),
    "mp_lstm_layer_fwd": (_I, [C.POINTER(LstmLayerDesc), _P, _P, _P, _P, _P, _P, _P, _P, _P, _SZ, _P]),
    "mp_lstm_layer_bwd": (_I, [C.POINTER(LstmLayerDesc), _P, _P, _P, _P, _P, _P, _P, _SZ, _P]),
    "mp_cast_f32_to_f16": (_I, [_SZ, _P, _P, _P]),
    "mp_fill_u32": (_I, [_SZ, C.c_uint32, _P, _P]),
    "mp_mfma_sustained_rate": (_I, [_P, _SZ, _P, _SZ, _I, _I, C.POINTER(C.c_double), _P]),
    "mp_unscale_check_update": (_I, [C.POINTER(TensorDesc), _I, C.POINTER(OptCfg), _P, _I, _P]),
}

_lib = None


def load() -> C.CDLL:
    """Load the HIP library.  There is no fallback: without libmp.so nothing in this package computes."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_1805_10387_amd.build` "
                               "(hipcc, gfx950). There is no CPU or PyTorch fallback.")
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib
