"""CPU oracle package -- TEST INFRASTRUCTURE ONLY (tests, smoke check, benchmark CPU baseline).

`apb_oracle` holds the numpy implementation; `capi` wraps the plain-C loops of
`apb_oracle_c.c` (built with gcc by `build_c()`), used where full-size layers
must finish in seconds.  Nothing in here imports the product package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

from . import apb_oracle  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "apb_oracle_c.c")
_LIB = os.path.join(_HERE, "libapb_oracle.so")
_lib: Optional[ctypes.CDLL] = None


def build_c(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build_c())
        _lib.apb_oracle_c_max_threads.restype = ctypes.c_int
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


class capi:
    """Thin ctypes wrappers; every array is C-contiguous numpy of the documented dtype."""

    @staticmethod
    def max_threads() -> int:
        return int(_load().apb_oracle_c_max_threads())

    @staticmethod
    def int_unpacked(bit: np.ndarray, c: np.ndarray) -> np.ndarray:
        bit8 = np.ascontiguousarray(bit, dtype=np.uint8)
        c8 = np.ascontiguousarray(c, dtype=np.int8)
        N, K = bit8.shape
        M = c8.shape[1]
        D = np.empty((N, M), dtype=np.int32)
        _load().apb_oracle_c_int_unpacked(_p(bit8), _p(c8), N, K, M, _p(D))
        return D

    @staticmethod
    def int_packed(sign_words: np.ndarray, packed: np.ndarray, K: int, M: int, bits: int,
                   threads: int = 1) -> np.ndarray:
        sw = np.ascontiguousarray(sign_words, dtype=np.uint32)
        pk = np.ascontiguousarray(packed, dtype=np.uint32)
        N = sw.shape[0]
        D = np.empty((N, M), dtype=np.int32)
        _load().apb_oracle_c_int_packed(_p(sw), _p(pk), N, K, M, bits, _p(D), threads)
        return D

    @staticmethod
    def sparse(row_ptr, col_idx, val, c: np.ndarray, step, threads: int = 1) -> np.ndarray:
        rp = np.ascontiguousarray(row_ptr, dtype=np.int32)
        ci = np.ascontiguousarray(col_idx, dtype=np.int32)
        v = np.ascontiguousarray(val, dtype=np.float32)
        c8 = np.ascontiguousarray(c, dtype=np.int8)
        N, M = len(rp) - 1, c8.shape[1]
        R = np.empty((N, M), dtype=np.float64)
        _load().apb_oracle_c_sparse(_p(rp), _p(ci), _p(v), _p(c8), ctypes.c_float(float(step)), N, M,
                                    _p(R), threads)
        return R

    @staticmethod
    def epilogue(alpha, step, D: np.ndarray, R: np.ndarray) -> np.ndarray:
        D = np.ascontiguousarray(D, dtype=np.int32)
        R = np.ascontiguousarray(R, dtype=np.float64)
        Y = np.empty(D.shape, dtype=np.float32)
        _load().apb_oracle_c_epilogue(ctypes.c_float(float(alpha)), ctypes.c_float(float(step)), _p(D), _p(R),
                                      ctypes.c_size_t(D.size), _p(Y))
        return Y

    @staticmethod
    def forward(layer: dict, packed: np.ndarray, c: np.ndarray, bits: int, step, threads: int = 1) -> dict:
        sw = np.ascontiguousarray(layer["sign_words"], dtype=np.uint32)
        rp = np.ascontiguousarray(layer["row_ptr"], dtype=np.int32)
        ci = np.ascontiguousarray(layer["col_idx"], dtype=np.int32)
        v = np.ascontiguousarray(layer["val"], dtype=np.float32)
        pk = np.ascontiguousarray(packed, dtype=np.uint32)
        c8 = np.ascontiguousarray(c, dtype=np.int8)
        N, K, M = layer["N"], layer["K"], c8.shape[1]
        D = np.empty((N, M), dtype=np.int32)
        R = np.empty((N, M), dtype=np.float64)
        Y = np.empty((N, M), dtype=np.float32)
        _load().apb_oracle_c_forward(_p(sw), _p(rp), _p(ci), _p(v), ctypes.c_float(float(layer["alpha"])),
                                     _p(pk), _p(c8), N, K, M, bits, ctypes.c_float(float(step)),
                                     _p(D), _p(R), _p(Y), threads)
        return {"D": D, "R": R, "Y": Y}
