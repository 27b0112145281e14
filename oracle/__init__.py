"""CPU oracle for the f16 GEMM hot path -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this package; the product (`paper_2108_13191_amd`) never does, and the two
share no code.  The arithmetic lives in `oracle_gemm.c` (plain C, binary64);
this file only builds that C file with gcc and marshals numpy arrays to it.

What is computed (paper, Evaluation section: C = A B + C, row-major; Listing
"Naive affine matmul"): C_ref = C0 + sum_k A[i,k] B[k,j] in binary64 in
increasing k, and S = sum_k |A[i,k]| |B[k,j]|.  The fused epilogue (bias
addition named in the paper's Background section, subsection Tensor Cores, as
the fusion that needs the accumulators' thread-data mapping) is the two plain
numpy lines of `bias_act`.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle_gemm.c")
_LIB = os.path.join(_HERE, "liboracle_gemm.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile oracle_gemm.c into liboracle_gemm.so with gcc (host only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, vp = ctypes.c_int64, ctypes.c_void_p
        lib.oracle_gemm_f16_rows.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64,
                                             ctypes.c_int, vp, i64, vp, vp]
        lib.oracle_gemm_f16_rows.restype = ctypes.c_int
        lib.oracle_gemm_f16.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64,
                                        ctypes.c_int, vp, vp]
        lib.oracle_gemm_f16.restype = ctypes.c_int
        for name in ("oracle_f16_bits_to_f64_array", "oracle_f64_to_f16_bits_array",
                     "oracle_f64_to_f32_bits_array"):
            getattr(lib, name).argtypes = [vp, vp, i64]
            getattr(lib, name).restype = None
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    """Threads the oracle's row loop runs on."""
    return int(_load().oracle_num_threads())


def _pitch(x: np.ndarray) -> int:
    if x.ndim != 2:
        raise ValueError("expected a 2-D array")
    if x.size == 0:
        return max(x.shape[1], 1)
    if x.shape[1] > 1 and x.strides[1] != x.itemsize:
        raise ValueError("rows must be contiguous")
    if x.shape[0] > 1:
        if x.strides[0] % x.itemsize:
            raise ValueError("row pitch must be a whole number of elements")
        return x.strides[0] // x.itemsize
    return max(x.shape[1], 1)


def gemm_f16(A: np.ndarray, B: np.ndarray, C0: np.ndarray, rows=None):
    """Oracle result for C0 + A @ B.

    A (M x K) and B (K x N) are numpy float16, C0 (M x N) is float32 (the
    f32-accumulate mode) or float16 (the f16-accumulate mode); rows may be
    strided views (row pitch > row length).  `rows`, if given, selects the
    output rows to evaluate.  Returns (C_ref, S), both float64, shape
    (len(rows) or M, N).
    """
    lib = _load()
    if A.dtype != np.float16 or B.dtype != np.float16:
        raise TypeError("A and B must be float16")
    if C0.dtype not in (np.float32, np.float16):
        raise TypeError("C0 must be float32 or float16")
    M, K = A.shape
    K2, N = B.shape
    if K2 != K or C0.shape != (M, N):
        raise ValueError("shape mismatch")
    lda = max(_pitch(A), K)
    ldb = max(_pitch(B), N)
    ldc = max(_pitch(C0), N)
    if rows is None:
        rows_arr, nrows, rows_p = None, M, None
    else:
        rows_arr = np.ascontiguousarray(rows, dtype=np.int64)
        nrows, rows_p = rows_arr.size, rows_arr.ctypes.data
    Cref = np.zeros((nrows, N), dtype=np.float64)
    S = np.zeros((nrows, N), dtype=np.float64)
    rc = lib.oracle_gemm_f16_rows(M, N, K, A.ctypes.data, lda, B.ctypes.data, ldb,
                                  C0.ctypes.data, ldc, int(C0.dtype == np.float16),
                                  rows_p, nrows, Cref.ctypes.data, S.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"oracle_gemm_f16_rows failed with code {rc}")
    return Cref, S


def bias_act(Cref: np.ndarray, bias=None, relu: bool = False) -> np.ndarray:
    """act(C_ref + bias[j]) in binary64: the per-column bias (any float dtype,
    widened exactly) is added to every row; ReLU is x < 0 ? 0 : x, so NaN and
    -0 pass through.  Cref is the binary64 output of gemm_f16."""
    out = np.array(Cref, dtype=np.float64, copy=True)
    if bias is not None:
        out = out + np.asarray(bias).astype(np.float64)[None, :]
    if relu:
        out = np.where(out < 0.0, 0.0, out)
    return out


def gemm_f16_rounding_every_slice(A: np.ndarray, B: np.ndarray, C0: np.ndarray, slice_k: int = 16) -> np.ndarray:
    """A literal reading of the paper's half-precision mode (section Half Precision
    Performance: the accumulation is done in binary16 too): the running sum is a
    binary16 value, and each slice of `slice_k` products (16 = the depth of the
    paper's m16n16k16 operation) is added to it exactly and the sum rounded to
    nearest even.  NOT the parity reference -- the library accumulates the whole
    k range in binary32 and rounds once, which `round_to_f16(gemm_f16(...)[0])`
    describes; this function exists to put a number on the difference between
    the two readings.  Returns binary64 values that are binary16-representable."""
    A64, B64 = np.asarray(A, np.float16).astype(np.float64), np.asarray(B, np.float16).astype(np.float64)
    acc = np.asarray(C0, np.float16).astype(np.float64)
    K = A64.shape[1]
    for k0 in range(0, K, slice_k):
        # <= slice_k products of 22-bit significands: the binary64 sum is exact to far below half a binary16 ulp
        acc = round_to_f16(acc + A64[:, k0:k0 + slice_k] @ B64[k0:k0 + slice_k, :]).astype(np.float64)
    return acc


def f16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Decode binary16 bit patterns (uint16) to float64 with the oracle's decoder."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.empty(bits.shape, dtype=np.float64)
    _load().oracle_f16_bits_to_f64_array(bits.ctypes.data, out.ctypes.data, bits.size)
    return out


def round_to_f16(x: np.ndarray) -> np.ndarray:
    """Round float64 to float16 once, ties to even (the oracle's encoder)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    out = np.empty(x.shape, dtype=np.uint16)
    _load().oracle_f64_to_f16_bits_array(x.ctypes.data, out.ctypes.data, x.size)
    return out.view(np.float16)


def round_to_f32(x: np.ndarray) -> np.ndarray:
    """Round float64 to float32 once, ties to even (the oracle's encoder)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    out = np.empty(x.shape, dtype=np.uint32)
    _load().oracle_f64_to_f32_bits_array(x.ctypes.data, out.ctypes.data, x.size)
    return out.view(np.float32)
