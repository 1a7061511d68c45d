"""ctypes front end of the fp64 CPU oracle (``lora_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, the smoke check and the benchmark's ``cpu_baseline`` leg may import this package;
it imports nothing from the HIP package and the HIP package never imports it.  All arithmetic
lives in the C file; this module only marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lora_oracle.c")
_LIB = os.path.join(_HERE, "liblora_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over tokens)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", _LIB, _SRC])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        for name in ("oracle_lora_shrink", "oracle_lora_expand", "oracle_lora_apply"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError("bf16 inputs are passed as uint16 bit patterns")
    return a


def _ptr_table(arrs: Sequence[Optional[np.ndarray]]):
    tab = (ctypes.c_void_p * len(arrs))()
    for i, a in enumerate(arrs):
        tab[i] = a.ctypes.data if a is not None else None
    return tab


def _prep(ranks, token_adapter, rows, T):
    ranks = np.ascontiguousarray(ranks, dtype=np.int32)
    ta = np.ascontiguousarray(token_adapter, dtype=np.int32)
    if rows is None:
        n_rows, rows_p, rows_a = T, None, None
    else:
        rows_a = np.ascontiguousarray(rows, dtype=np.int32)
        if rows_a.size and (rows_a.min() < 0 or rows_a.max() >= T):
            raise ValueError("row index out of range")
        n_rows, rows_p = int(rows_a.size), rows_a.ctypes.data_as(ctypes.c_void_p)
    return ranks, ta, n_rows, rows_p, rows_a


def _check_adapters(mats, ranks, ta, want_shape):
    used = np.unique(ta)
    for a in used[used >= 0]:
        if a >= len(mats) or mats[a] is None:
            raise ValueError(f"adapter {a} is routed to but has no weights")
        if mats[a].shape != want_shape(int(ranks[a])):
            raise ValueError(f"adapter {a}: shape {mats[a].shape} != {want_shape(int(ranks[a]))}")


def lora_shrink(x_bits, token_adapter, ranks, A: Sequence[Optional[np.ndarray]], rows=None) -> np.ndarray:
    """v [n_rows][max rank] fp64 (zero beyond each token's rank).  A[a] is bf16 bits [in][r_a]."""
    x = _u16(x_bits)
    T, in_f = x.shape
    ranks, ta, n_rows, rows_p, _keep = _prep(ranks, token_adapter, rows, T)
    A = [None if m is None else _u16(m) for m in A]
    _check_adapters(A, ranks, ta, lambda r: (in_f, r))
    stride = int(ranks.max()) if ranks.size else 1
    v = np.zeros((n_rows, stride), dtype=np.float64)
    rc = _load().oracle_lora_shrink(n_rows, rows_p, in_f, x.ctypes.data_as(ctypes.c_void_p),
                                    ta.ctypes.data_as(ctypes.c_void_p), len(A),
                                    ranks.ctypes.data_as(ctypes.c_void_p), _ptr_table(A),
                                    v.ctypes.data_as(ctypes.c_void_p), stride)
    if rc:
        raise RuntimeError("oracle_lora_shrink rejected its arguments")
    return v


def lora_expand(v, token_adapter, ranks, scales, B: Sequence[Optional[np.ndarray]], out_features: int,
                y0=None, rows=None) -> np.ndarray:
    """y [n_rows][out] fp64 from a given v [n_rows][stride] (fp64).  B[a] is bf16 bits [r_a][out]."""
    v = np.ascontiguousarray(v, dtype=np.float64)
    ta_full = np.ascontiguousarray(token_adapter, dtype=np.int32)
    ranks, ta, n_rows, rows_p, _keep = _prep(ranks, ta_full, rows, ta_full.shape[0])
    if v.shape[0] != n_rows:
        raise ValueError("v has one row per evaluated token")
    scales = np.ascontiguousarray(scales, dtype=np.float32)
    B = [None if m is None else _u16(m) for m in B]
    _check_adapters(B, ranks, ta, lambda r: (r, out_features))
    y0p = None
    if y0 is not None:
        y0 = np.ascontiguousarray(y0, dtype=np.float64)
        assert y0.shape == (n_rows, out_features)
        y0p = y0.ctypes.data_as(ctypes.c_void_p)
    y = np.empty((n_rows, out_features), dtype=np.float64)
    rc = _load().oracle_lora_expand(n_rows, rows_p, out_features, v.ctypes.data_as(ctypes.c_void_p),
                                    int(v.shape[1]), ta.ctypes.data_as(ctypes.c_void_p), len(B),
                                    ranks.ctypes.data_as(ctypes.c_void_p),
                                    scales.ctypes.data_as(ctypes.c_void_p), _ptr_table(B), y0p,
                                    y.ctypes.data_as(ctypes.c_void_p))
    if rc:
        raise RuntimeError("oracle_lora_expand rejected its arguments")
    return y


def lora_apply(x_bits, token_adapter, ranks, scales, A: Sequence[Optional[np.ndarray]],
               B: Sequence[Optional[np.ndarray]], y0=None, rows=None) -> np.ndarray:
    """y [n_rows][out] fp64 = y0 + s_a (x A_a) B_a per token; rows without adapter return y0.

    x_bits: uint16 [T][in]; A[a]: uint16 [in][r_a]; B[a]: uint16 [r_a][out]; y0: fp64 [n_rows][out] or None.
    """
    x = _u16(x_bits)
    T, in_f = x.shape
    ranks, ta, n_rows, rows_p, _keep = _prep(ranks, token_adapter, rows, T)
    if ta.shape[0] != T:
        raise ValueError("token_adapter has one entry per row of x")
    scales = np.ascontiguousarray(scales, dtype=np.float32)
    A = [None if m is None else _u16(m) for m in A]
    B = [None if m is None else _u16(m) for m in B]
    out_f = next((m.shape[1] for m in B if m is not None), None)
    if out_f is None:  # no adapter given at all (no token uses one): the width of y comes from y0
        if y0 is None:
            raise ValueError("no adapter and no y0: the width of y is not defined")
        out_f = int(np.shape(y0)[1])
    _check_adapters(A, ranks, ta, lambda r: (in_f, r))
    _check_adapters(B, ranks, ta, lambda r: (r, out_f))
    y0p = None
    if y0 is not None:
        y0 = np.ascontiguousarray(y0, dtype=np.float64)
        assert y0.shape == (n_rows, out_f)
        y0p = y0.ctypes.data_as(ctypes.c_void_p)
    y = np.empty((n_rows, out_f), dtype=np.float64)
    rc = _load().oracle_lora_apply(n_rows, rows_p, in_f, out_f, x.ctypes.data_as(ctypes.c_void_p),
                                   ta.ctypes.data_as(ctypes.c_void_p), len(A),
                                   ranks.ctypes.data_as(ctypes.c_void_p),
                                   scales.ctypes.data_as(ctypes.c_void_p), _ptr_table(A), _ptr_table(B),
                                   y0p, y.ctypes.data_as(ctypes.c_void_p))
    if rc:
        raise RuntimeError("oracle_lora_apply rejected its arguments")
    return y


def lora_linear(x_bits, W_bits, token_adapter, ranks, scales, A: Sequence[Optional[np.ndarray]],
                B: Sequence[Optional[np.ndarray]], rows=None) -> np.ndarray:
    """y [n_rows][out] fp64 = x W + s_a (x A_a) B_a per token (rows without adapter: x W).

    x_bits: uint16 [T][in]; W_bits: uint16 [in][out]; A[a]: uint16 [in][r_a]; B[a]: uint16 [r_a][out].
    """
    x = _u16(x_bits)
    W = _u16(W_bits)
    T, in_f = x.shape
    if W.ndim != 2 or W.shape[0] != in_f:
        raise ValueError("W is [in][out]")
    out_f = int(W.shape[1])
    ranks, ta, n_rows, rows_p, _keep = _prep(ranks, token_adapter, rows, T)
    if ta.shape[0] != T:
        raise ValueError("token_adapter has one entry per row of x")
    scales = np.ascontiguousarray(scales, dtype=np.float32)
    A = [None if m is None else _u16(m) for m in A]
    B = [None if m is None else _u16(m) for m in B]
    _check_adapters(A, ranks, ta, lambda r: (in_f, r))
    _check_adapters(B, ranks, ta, lambda r: (r, out_f))
    y = np.empty((n_rows, out_f), dtype=np.float64)
    rc = _load().oracle_lora_linear(n_rows, rows_p, in_f, out_f, x.ctypes.data_as(ctypes.c_void_p),
                                    W.ctypes.data_as(ctypes.c_void_p), ta.ctypes.data_as(ctypes.c_void_p), len(A),
                                    ranks.ctypes.data_as(ctypes.c_void_p), scales.ctypes.data_as(ctypes.c_void_p),
                                    _ptr_table(A), _ptr_table(B), y.ctypes.data_as(ctypes.c_void_p))
    if rc:
        raise RuntimeError("oracle_lora_linear rejected its arguments")
    return y


def threads() -> int:
    """OpenMP threads the oracle will use (for the benchmark's 'cores' field)."""
    lib = _load()
    try:
        gomp = ctypes.CDLL("libgomp.so.1")
        gomp.omp_get_max_threads.restype = ctypes.c_int
        return int(gomp.omp_get_max_threads())
    except OSError:
        del lib
        return len(os.sched_getaffinity(0))
