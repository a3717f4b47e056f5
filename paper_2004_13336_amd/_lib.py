"""ctypes loader for libshardupdate.so.  There is no fallback: without the HIP library nothing runs."""
from __future__ import annotations

import ctypes as C
import os

from .build import LIB_PATH, build_library

_lib = None


class ShardError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = "unknown"
        try:
            msg = lib().shard_strerror(status).decode()
        except Exception:
            pass
        super().__init__("%s failed: %s (status %d)" % (where, msg, status))


class AdamHP(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float)]


class MomentumHP(C.Structure):
    _fields_ = [("lr", C.c_float), ("mu", C.c_float), ("weight_decay", C.c_float)]


class LambHP(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float)]


class LarsHP(C.Structure):
    _fields_ = [("lr", C.c_float), ("mu", C.c_float), ("weight_decay", C.c_float), ("trust_coeff", C.c_float),
                ("eps", C.c_float)]


class AdafactorHP(C.Structure):
    _fields_ = [("eps1", C.c_float), ("eps2", C.c_float), ("clip_threshold", C.c_float),
                ("decay_exponent", C.c_float), ("max_rho", C.c_float)]


_P = C.c_void_p
_I64P = C.POINTER(C.c_int64)
_IP = C.POINTER(C.c_int)
_DP = C.POINTER(C.c_double)

# name -> (restype, argtypes); mirrors include/shardupdate.h declaration by declaration
SIGNATURES = {
    "shard_strerror": (C.c_char_p, [C.c_int]),
    "shard_kernel_name": (C.c_char_p, [C.c_int]),
    "shard_plan": (C.c_int, [C.c_int, _I64P, C.c_int, C.c_int, C.POINTER(C.c_uint32), C.c_int, C.POINTER(_P)]),
    "shard_plan_rows": (C.c_int, [C.c_int, _I64P, _I64P, C.c_int, C.c_int, C.POINTER(C.c_uint32), C.c_int, C.POINTER(_P)]),
    "shard_plan_info": (C.c_int, [_P, _I64P, _I64P, _I64P, C.POINTER(C.c_int), C.POINTER(C.c_size_t)]),
    "shard_plan_segments": (C.c_int, [_P, _I64P, _I64P]),
    "shard_plan_real_count": (C.c_int, [_P, C.c_int, _I64P]),
    "shard_plan_bind": (C.c_int, [_P, _P, C.c_size_t, _P]),
    "shard_plan_free": (None, [_P]),
    "shard_format": (C.c_int, [_P, C.c_int, C.POINTER(_P), C.c_int, _P, C.c_int, _P]),
    "unshard_format": (C.c_int, [_P, _P, C.c_int64, C.c_int, C.POINTER(_P), C.c_int, _P]),
    "shard_update_adam": (C.c_int, [_P, C.c_int, _P, _P, _P, _P, _P, C.POINTER(AdamHP), C.c_int64, _P]),
    "shard_update_momentum": (C.c_int, [_P, C.c_int, _P, _P, _P, _P, C.POINTER(MomentumHP), _P]),
    "shard_update_lamb_partials": (C.c_int, [_P, C.c_int, _P, _P, _P, _P, C.POINTER(LambHP), C.c_int64, _P, _P]),
    "shard_update_lamb_apply": (C.c_int, [_P, C.c_int, _P, _P, _P, _P, C.POINTER(LambHP), C.c_int64, _P, _P]),
    "shard_update_lamb": (C.c_int, [_P, C.c_int, _P, _P, _P, _P, _P, C.POINTER(LambHP), C.c_int64, _P, _P, _P]),
    "shard_update_lamb_noalloc": (C.c_int, [_P, C.c_int, _P, _P, _P, _P, _P, C.POINTER(LambHP), C.c_int64, _P, _P, _P]),
    "shard_update_adam_full_grads": (C.c_int, [_P, C.c_int, _P, C.POINTER(_P), C.c_int, _P, _P, _P, C.POINTER(AdamHP),
                                               C.c_int64, _P]),
    "shard_update_momentum_full_grads": (C.c_int, [_P, C.c_int, _P, C.POINTER(_P), C.c_int, _P, _P,
                                                   C.POINTER(MomentumHP), _P]),
    "shard_update_lamb_partials_full_grads": (C.c_int, [_P, C.c_int, _P, C.POINTER(_P), C.c_int, _P, _P,
                                                        C.POINTER(LambHP), C.c_int64, _P, _P]),
    "shard_update_lamb_full_grads": (C.c_int, [_P, C.c_int, _P, C.POINTER(_P), C.c_int, _P, _P, _P, C.POINTER(LambHP),
                                               C.c_int64, _P, _P, _P]),
    "shard_update_lars_partials_full_grads": (C.c_int, [_P, C.c_int, _P, C.POINTER(_P), C.c_int, _P, _P]),
    "shard_update_lars_apply_full_grads": (C.c_int, [_P, C.c_int, _P, C.POINTER(_P), C.c_int, _P, _P,
                                                     C.POINTER(LarsHP), _P, _P]),
    "shard_update_lars_full_grads": (C.c_int, [_P, C.c_int, _P, C.POINTER(_P), C.c_int, _P, _P, C.POINTER(LarsHP), _P,
                                               _P, _P]),
    "shard_format_all": (C.c_int, [_P, C.POINTER(_P), C.c_int, _P, C.c_int64, C.c_int, _P]),
    "shard_update_lars_partials": (C.c_int, [_P, C.c_int, _P, _P, _P, _P]),
    "shard_update_lars_apply": (C.c_int, [_P, C.c_int, _P, _P, _P, _P, C.POINTER(LarsHP), _P, _P]),
    "shard_update_lars": (C.c_int, [_P, C.c_int, _P, _P, _P, _P, C.POINTER(LarsHP), _P, _P, _P]),
    "shard_plan_rowcol_layout": (C.c_int, [_P, _I64P, _I64P, _I64P, _I64P]),
    "shard_reduce_sq_rows_cols": (C.c_int, [_P, C.c_int, _P, _P, _P, _P]),
    "shard_update_adafactor_partials": (C.c_int, [_P, C.c_int, _P, _P, _P, _P, _P, _P, _P]),
    "shard_update_adafactor_moments": (C.c_int, [_P, C.c_int, _P, _P, _P, _P, _P, _P, C.POINTER(AdafactorHP), C.c_int64, _P, _P]),
    "shard_update_adafactor_apply": (C.c_int, [_P, C.c_int, _P, _P, _P, _P, _P, C.POINTER(AdafactorHP), C.c_int64, _P]),
    "shard_update_adafactor": (C.c_int, [_P, C.c_int, _P, _P, _P, _P, _P, C.POINTER(AdafactorHP), C.c_int64, _P, _P, _P, _P]),
    "shard_partial_sharding": (C.c_int, [C.c_int, C.c_int, C.c_int, _IP, _IP, _IP, _IP]),
    "shard_two_phase_shard_id": (C.c_int, [C.c_int, C.c_int, C.c_int, _IP]),
    "shard_concat_partition": (C.c_int, [C.c_int64, C.c_int, C.c_int, _I64P, _I64P]),
    "shard_peak_memory": (C.c_int, [C.c_double, C.c_double, C.c_double, C.c_int, _DP, _DP]),
    "shard_plan_peak_bytes": (C.c_int, [_P, C.c_int, C.c_int, C.c_int64, _I64P, _I64P]),
    "shard_profile_enable": (C.c_int, [_P, C.c_int]),
    "shard_profile_read": (C.c_int, [_P, C.c_int, _I64P, C.POINTER(C.c_double)]),
    "shard_profile_reset": (C.c_int, [_P]),
    "shard_profile_plain_copy": (C.c_int, [_P, _P, _P, C.c_size_t, _P]),
    "shard_profile_adam_shape": (C.c_int, [_P, _P, _P, _P, _P, C.POINTER(AdamHP), C.c_int64, C.c_int, C.c_int, _P]),
    "shard_plan_release_captured_tables": (C.c_int, [_P]),
    "shard_plan_set_copy_walk": (C.c_int, [_P, C.c_int]),
    "shard_plan_copy_walk": (C.c_int, [_P, C.c_int, _P, C.POINTER(C.c_int), C.POINTER(C.c_float)]),
    "shard_plan_tune_copy_walk": (C.c_int, [_P, C.c_int, _P, C.c_int64, C.c_int, C.POINTER(_P), C.c_int, _P,
                                            C.POINTER(C.c_int), C.POINTER(C.c_float)]),
}


def lib() -> C.CDLL:
    """The loaded library; built in-tree first if no built library is there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            build_library()
        handle = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(handle, name)          # AttributeError if the library lacks a declared symbol
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib
