"""Thin ctypes binding of the C ABI in include/gemm_f16.h.

Argument marshalling only: every step of the GEMM runs in the HIP kernels of
libgemm_f16.so.  There is no fallback: if the library has not been built (run
`python -m paper_2108_13191_amd.build`), loading raises.
Functions take raw device pointers (ints) or objects with `data_ptr()` (torch
tensors); nothing here computes.
"""
from __future__ import annotations

import ctypes
import os

import contextlib

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgemm_f16.so")
# the same library plus the comparison kernels and ablation rows (never selected; reached by
# forcing their configuration ids, which follow the product's): see build.py
LADDER_LIB_PATH = os.path.join(_HERE, "libgemm_f16_ladder.so")
_libs = {}
_active = "product"


@contextlib.contextmanager
def library(kind: str):
    """Within the block every function of this module calls into the named build
    ("product" or "ladder").  The two keep separate forced-configuration state."""
    global _active
    prev, _active = _active, kind
    try:
        yield
    finally:
        _active = prev

OK = 0
ERR_SIZE, ERR_PITCH, ERR_NULL, ERR_LAUNCH, ERR_CONFIG, ERR_ALIGN, ERR_WORKSPACE = -1, -2, -3, -4, -5, -6, -7


class GemmConfig(ctypes.Structure):
    _fields_ = [("id", ctypes.c_int32), ("block_m", ctypes.c_int32), ("block_n", ctypes.c_int32),
                ("block_k", ctypes.c_int32), ("waves", ctypes.c_int32), ("wave_m", ctypes.c_int32),
                ("wave_n", ctypes.c_int32), ("lds_bytes", ctypes.c_int32), ("grid", ctypes.c_int64),
                ("split_rows", ctypes.c_int32), ("id2", ctypes.c_int32), ("name", ctypes.c_char * 48)]

    def as_dict(self):
        d = {k: getattr(self, k) for k, _ in self._fields_}
        d["name"] = self.name.decode()
        return d


class GemmError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        super().__init__(f"gemm_f16 error {code}: {strerror(code)}")


def load() -> ctypes.CDLL:
    """Load the active library (built in-tree); raise if it is missing."""
    if _active not in _libs:
        path = {"product": LIB_PATH, "ladder": LADDER_LIB_PATH}[_active]
        if not os.path.exists(path):
            raise ImportError(
                f"{path} is missing: build the HIP library first "
                "(python -m paper_2108_13191_amd.build); there is no CPU fallback")
        lib = ctypes.CDLL(path)
        i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        for name in ("gemm_f16_f32acc", "gemm_f16_f16acc", "gemm_f16_f16acc_static_workspace"):
            f = getattr(lib, name)
            f.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, vp]
            f.restype = ci
        for name in ("gemm_f16_f32acc_bias_act", "gemm_f16_f16acc_bias_act"):
            f = getattr(lib, name)
            f.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, vp, ci, vp]
            f.restype = ci
        lib.gemm_f16_f16acc_workspace_bytes.argtypes = [i64, i64, i64]
        lib.gemm_f16_f16acc_workspace_bytes.restype = i64
        lib.gemm_f16_f16acc_workspace.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, vp, i64, vp]
        lib.gemm_f16_f16acc_workspace.restype = ci
        lib.gemm_strerror.argtypes = [ci]
        lib.gemm_strerror.restype = ctypes.c_char_p
        lib.gemm_f16_query_config.argtypes = [ci, i64, i64, i64, vp, i64, vp, i64, vp, i64,
                                              ctypes.POINTER(GemmConfig)]
        lib.gemm_f16_query_config.restype = ci
        lib.gemm_f16_num_configs.argtypes = []
        lib.gemm_f16_num_configs.restype = ci
        lib.gemm_f16_describe_config.argtypes = [ci, ctypes.POINTER(GemmConfig)]
        lib.gemm_f16_describe_config.restype = ci
        lib.gemm_f16_force_config.argtypes = [ci]
        lib.gemm_f16_force_config.restype = ci
        _libs[_active] = lib
    return _libs[_active]


def _ptr(x) -> int:
    if x is None:
        return 0
    if hasattr(x, "data_ptr"):
        return int(x.data_ptr())
    return int(x)


def gemm_f16_f32acc(M, N, K, A, lda, B, ldb, C, ldc, stream=0) -> int:
    """C (f32) += A (f16) @ B (f16); returns the library's status code."""
    return load().gemm_f16_f32acc(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, _ptr(stream))


def gemm_f16_f16acc(M, N, K, A, lda, B, ldb, C, ldc, stream=0) -> int:
    """C (f16) += A (f16) @ B (f16), f32 accumulation, one rounding on store."""
    return load().gemm_f16_f16acc(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, _ptr(stream))


def gemm_f16_f16acc_workspace_bytes(M, N, K) -> int:
    """Bytes of workspace that let gemm_f16_f16acc_workspace cut this problem along k (0: none needed)."""
    return load().gemm_f16_f16acc_workspace_bytes(M, N, K)


def gemm_f16_f16acc_workspace(M, N, K, A, lda, B, ldb, C, ldc, workspace, workspace_bytes, stream=0) -> int:
    """gemm_f16_f16acc with caller-provided scratch memory (device, 16-byte aligned) for split-k plans."""
    return load().gemm_f16_f16acc_workspace(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, _ptr(workspace), workspace_bytes, _ptr(stream))


def gemm_f16_f16acc_static_workspace(M, N, K, A, lda, B, ldb, C, ldc, stream=0) -> int:
    """gemm_f16_f16acc_workspace on the library's own fixed scratch array: allocates nothing."""
    return load().gemm_f16_f16acc_static_workspace(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, _ptr(stream))


ACT_NONE, ACT_RELU = 0, 1


def gemm_f16_f32acc_bias_act(M, N, K, A, lda, B, ldb, C, ldc, bias, act, stream=0) -> int:
    """C (f32) = act(C + A @ B + bias[None, :]); bias f32 device vector or None."""
    return load().gemm_f16_f32acc_bias_act(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, _ptr(bias), act, _ptr(stream))


def gemm_f16_f16acc_bias_act(M, N, K, A, lda, B, ldb, C, ldc, bias, act, stream=0) -> int:
    """C (f16) = act(C + A @ B + bias[None, :]), f32 arithmetic, one rounding on store; bias f16 or None."""
    return load().gemm_f16_f16acc_bias_act(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, _ptr(bias), act, _ptr(stream))


def strerror(code: int) -> str:
    return load().gemm_strerror(code).decode()


def query_config(c_is_f16, M, N, K, A, lda, B, ldb, C, ldc) -> dict:
    out = GemmConfig()
    rc = load().gemm_f16_query_config(int(c_is_f16), M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc,
                                      ctypes.byref(out))
    if rc != OK:
        raise GemmError(rc)
    return out.as_dict()


def num_configs() -> int:
    return load().gemm_f16_num_configs()


def describe_config(cfg_id: int) -> dict:
    out = GemmConfig()
    rc = load().gemm_f16_describe_config(cfg_id, ctypes.byref(out))
    if rc != OK:
        raise GemmError(rc)
    return out.as_dict()


def force_config(cfg_id: int) -> int:
    return load().gemm_f16_force_config(cfg_id)


def check(rc: int) -> None:
    if rc != OK:
        raise GemmError(rc)
