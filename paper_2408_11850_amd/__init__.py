"""Thin ctypes binding of libspec.so (the gfx950 speculative-decoding library).

Argument marshalling only: every step of the decoding path runs in the library's HIP kernels.
PyTorch is used by callers for device memory and streams.  There is no CPU fallback: if the
library is missing or was not built, load_library() raises.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspec.so")

SPEC_OK, SPEC_E_INVAL, SPEC_E_NOMEM, SPEC_E_STATE, SPEC_E_HIP = 0, -1, -2, -3, -4
SPEC_TARGET, SPEC_DRAFT = 0, 1
SPEC_ACCEPT_AR, SPEC_ACCEPT_SD, SPEC_ACCEPT_PRE, SPEC_ACCEPT_POST, SPEC_ACCEPT_PRE_GUESS = 0, 1, 2, 3, 4
SPEC_MODE_PRE, SPEC_MODE_POST = 0, 1
SPEC_MAX_TOKENS = 32
PAGE_TOKENS = 64
ALGO_AR, ALGO_SD, ALGO_PEARL = 0, 1, 2
ALGO_PEARL_NO_PRE, ALGO_PEARL_NO_POST = 3, 4      # the two ablations
ALGO_PEARL_GUESS = 5                               # pre-verify steps cover several draft tokens (Section 4.3, closing remark)
SPEC_OPT_GEMM_WGS_PER_CU = 1
SPEC_OPT_GRAPHS = 2
SPEC_OPT_PREFILL = 3
SPEC_OPT_TEST_FAIL_PREFILL = 4
SPEC_OPT_FUSE_SINGLE = 5
SPEC_OPT_GUESS_TOKENS = 6
SPEC_OPT_TARGET_TAIL_LAYERS = 7
EPI_STORE, EPI_RESID, EPI_SWIGLU = 0, 1, 2


class ModelDesc(C.Structure):
    _fields_ = [("n_layers", C.c_int), ("d_model", C.c_int), ("n_heads", C.c_int), ("n_kv_heads", C.c_int),
                ("head_dim", C.c_int), ("d_ffn", C.c_int), ("vocab", C.c_int),
                ("rope_theta", C.c_float), ("rms_eps", C.c_float)]


class Weights(C.Structure):
    _fields_ = [("tok_embed", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p),
                ("attn_norm", C.POINTER(C.c_void_p)), ("wqkv", C.POINTER(C.c_void_p)),
                ("wo", C.POINTER(C.c_void_p)), ("ffn_norm", C.POINTER(C.c_void_p)),
                ("w_gateup", C.POINTER(C.c_void_p)), ("w_down", C.POINTER(C.c_void_p))]


class Config(C.Structure):
    _fields_ = [("gamma_max", C.c_int), ("max_seq", C.c_int), ("page_tokens", C.c_int),
                ("temperature", C.c_float), ("logit_scale", C.c_float),
                ("stream_target", C.c_void_p), ("stream_draft", C.c_void_p)]


# name -> (restype, argtypes); every symbol include/spec.h declares
_P = C.c_void_p
_PI = C.POINTER(C.c_int)
_PF = C.POINTER(C.c_float)
_PI32 = C.POINTER(C.c_int32)
SIGNATURES = {
    "spec_init": (C.c_int, [C.POINTER(Config), C.POINTER(ModelDesc), C.POINTER(Weights), C.POINTER(ModelDesc),
                            C.POINTER(Weights), C.POINTER(_P)]),
    "spec_free": (None, [_P]),
    "spec_prefill": (C.c_int, [_P, _PI32, C.c_int, C.c_int]),
    "spec_draft_step": (C.c_int, [_P, C.c_float, _PI32]),
    "spec_verify": (C.c_int, [_P, _PI32, C.c_int, _PF]),
    "spec_verify_guess": (C.c_int, [_P, _PI32, C.c_int, _PI, _PF]),
    "spec_accept": (C.c_int, [_P, C.c_int, _PF, C.c_int, C.c_float, C.c_longlong, _PI, _PI32, _PI, _PI, _PI]),
    "spec_rollback_kv": (C.c_int, [_P, C.c_int, C.c_int]),
    "spec_drop_drafts": (C.c_int, [_P]),
    "spec_rewind": (C.c_int, [_P, C.c_int]),
    "spec_kv_len": (C.c_int, [_P, C.c_int]),
    "spec_pending_rows": (C.c_int, [_P]),
    "spec_committed_len": (C.c_int, [_P]),
    "spec_kv_free_pages": (C.c_int, [_P, C.c_int]),
    "spec_forward_count": (C.c_longlong, [_P, C.c_int]),
    "spec_generate": (C.c_int, [_P, C.c_int, C.c_int, C.c_int, C.c_int, _PF, _PF, _PF, C.POINTER(C.c_uint8), _PI32,
                                C.POINTER(C.c_double)]),
    "spec_calibrate_gamma": (C.c_int, [_P, C.c_int, C.c_int, C.c_int, _PI, C.POINTER(C.c_double),
                                       C.POINTER(C.c_double)]),
    "spec_last_error": (C.c_char_p, []),
    "spec_pack_weight": (C.c_int, [_P, _P, C.c_int, C.c_int, C.c_int, C.c_int, _P]),
    "spec_packed_bytes": (C.c_size_t, [C.c_int, C.c_int]),
    "spec_gemm_plan_query": (C.c_int, [C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int)]),
    "spec_gemm": (C.c_int, [_P, _P, _P, C.c_int, C.c_int, C.c_int, _P, _P]),
    "spec_gemm_workspace_bytes": (C.c_size_t, [C.c_int, C.c_int, C.c_int]),
    "spec_gemm_partials": (C.c_int, [_P, _P, C.c_int, C.c_int, C.c_int, _P, _P]),
    "spec_dense_gemm": (C.c_int, [_P, _P, _P, _P, C.c_int, C.c_int, C.c_int, C.c_int, _P]),
    "spec_read_probe": (C.c_int, [_P, C.c_size_t, _P, _P]),
    "spec_sample_row": (C.c_int, [_P, C.c_int, C.c_float, C.c_float, C.c_float, _P, _P, _P]),
    "spec_accept_rows": (C.c_int, [_P, C.c_int, _P, _P, C.c_int, C.c_int, C.c_float, C.c_float, _PF, C.c_float,
                                   _PI32, _P]),
    "spec_accept_rows_static": (C.c_int, [_P, C.c_int, _P, _P, C.c_int, C.c_int, C.c_float, C.c_float, _PF, C.c_float,
                                          _P, _P]),
    "spec_set_option": (C.c_int, [_P, C.c_int, C.c_int]),
    "spec_get_option": (C.c_int, [_P, C.c_int, _PI]),
    "spec_set_profile": (C.c_int, [_P, C.c_int]),
    "spec_profile_read": (C.c_int, [_P, C.POINTER(C.c_double), C.POINTER(C.c_longlong), C.POINTER(C.c_double)]),
}

_lib = None


class SpecError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libspec error {code}: {msg}")
        self.code = code


def load_library() -> C.CDLL:
    """Load libspec.so built in-tree (python __graft_entry__.py).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not found: build it with `python __graft_entry__.py` (there is no fallback)")
    lib = C.CDLL(LIB_PATH)
    for name, (res, args) in SIGNATURES.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def check(rc: int) -> int:
    if rc < 0:
        raise SpecError(rc, load_library().spec_last_error().decode())
    return rc


from .binding import SpecContext, pack_model, gemm, dense_gemm, sample_row, accept_rows, accept_rows_static, read_probe  # noqa: E402,F401
