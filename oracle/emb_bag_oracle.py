"""ctypes loader for the CPU oracle (`emb_bag_oracle.c`).  TEST INFRASTRUCTURE ONLY.

Only tests, `__graft_entry__.smoke()` and the `cpu_baseline` leg of `bench.py` may import this
module; the product path never does.  It imports nothing from the HIP package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "emb_bag_oracle.c")
LIB = os.path.join(_HERE, "liboracle_embbag.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, -O2, OpenMP over bags)."""
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               "-o", LIB, SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return LIB


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(LIB)
        lib.oracle_emb_bag.restype = ctypes.c_int
        lib.oracle_emb_bag.argtypes = [
            ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_set_num_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(int(n))


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def emb_bag(tables: np.ndarray, table_offsets: np.ndarray, indices: np.ndarray,
            offsets: np.ndarray, B: int, mode: str = "sum",
            weights: Optional[np.ndarray] = None,
            out_ld: int = 0, codes: str = "u8", strict: bool = False):
    """Reference output and error-bound scale, both fp64 [B, out_ld]; with `strict` also the
    strict bound scale, the sum of |w * element| with a quantised element taken as one number
    (scale * code + bias) rather than as the two terms an implementation adds.

    `codes` says what the bytes of a quantised (uint8) table stand for: "u8" unsigned integers,
    "fp8" OCP E4M3 8-bit floats.

    tables: [sum R_t, D] float32, float16 or uint16 (= bfloat16 bits) host array, or uint8
    [sum R_t, D + 8] (D codes, fp32 scale, fp32 bias per row: element = scale * code + bias); table_offsets int64 [T+1];
    indices int64 [NL]; offsets int64 [T*B+1]; weights float32 [NL] or None.
    Raises ValueError on the error codes of the C function.
    """
    if tables.ndim != 2:
        raise ValueError("tables must be [rows, D]")
    if tables.dtype == np.float32:
        dtype = 0
    elif tables.dtype == np.float16:
        dtype = 1
    elif tables.dtype == np.uint16:   # numpy has no bfloat16: raw bit patterns
        dtype = 2
    elif tables.dtype == np.uint8:    # row-wise quantised: D codes + fp32 scale + fp32 bias
        dtype = {"u8": 3, "fp8": 4}[codes]
        if tables.shape[1] <= 8:
            raise ValueError("quantised rows need D + 8 bytes")
    else:
        raise ValueError("tables must be float32, float16, uint16 (bfloat16 bits) or uint8 "
                         "(quantised rows)")
    tables = np.ascontiguousarray(tables)
    table_offsets = np.ascontiguousarray(table_offsets, dtype=np.int64)
    indices = np.ascontiguousarray(indices, dtype=np.int64)
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    if weights is not None:
        weights = np.ascontiguousarray(weights, dtype=np.float32)
        if len(weights) != len(indices):
            raise ValueError("weights and indices differ in length")
    T = len(table_offsets) - 1
    D = tables.shape[1] - 8 if dtype >= 3 else tables.shape[1]
    if len(offsets) != T * B + 1:
        raise ValueError("offsets must have T*B+1 entries")
    if int(offsets[-1]) != len(indices):
        raise ValueError("offsets[-1] must equal len(indices)")
    if int(table_offsets[-1]) > tables.shape[0]:
        raise ValueError("table_offsets exceed the arena")
    ld = out_ld if out_ld else T * D
    ref = np.zeros((B, ld), dtype=np.float64)
    bound = np.zeros((B, ld), dtype=np.float64)
    sbound = np.zeros((B, ld), dtype=np.float64) if strict else None
    rc = _load().oracle_emb_bag(T, B, D, dtype, {"sum": 0, "mean": 1, "max": 2}[mode], _ptr(tables),
                                _ptr(table_offsets), _ptr(indices), _ptr(offsets),
                                _ptr(weights), ld, _ptr(ref), _ptr(bound), _ptr(sbound))
    if rc != 0:
        raise ValueError({-1: "bad argument", -2: "offsets not monotone from 0",
                          -3: "index out of range"}.get(rc, f"oracle error {rc}"))
    return (ref, bound, sbound) if strict else (ref, bound)


def emb_bag_mixed(tables, indices: np.ndarray, offsets: np.ndarray, B: int, mode: str = "sum",
                  weights: Optional[np.ndarray] = None,
                  out_ld: int = 0, codes: str = "u8") -> Tuple[np.ndarray, np.ndarray]:
    """Tables of different widths: `tables` is a list of per-table host arrays ([R_t, D_t], or
    uint8 [R_t, D_t + 8] for quantised rows).  The definition is unchanged - bag (t, b) pools rows
    of table t - and table t's block starts at column sum of the widths before it; each table is
    evaluated on its own by `emb_bag`."""
    T = len(tables)
    dims = [a.shape[1] - 8 if a.dtype == np.uint8 else a.shape[1] for a in tables]
    total = int(sum(dims))
    ld = out_ld if out_ld else total
    if ld < total:
        raise ValueError("out_ld smaller than the sum of the widths")
    ref = np.zeros((B, ld), dtype=np.float64)
    bound = np.zeros((B, ld), dtype=np.float64)
    col = 0
    for t in range(T):
        o = np.asarray(offsets[t * B:(t + 1) * B + 1], dtype=np.int64)
        s, e = int(o[0]), int(o[-1])
        w = None if weights is None else weights[s:e]
        r, b = emb_bag(tables[t], np.array([0, tables[t].shape[0]], np.int64), indices[s:e], o - s,
                       B, mode, weights=w, codes=codes)
        ref[:, col:col + dims[t]] = r
        bound[:, col:col + dims[t]] = b
        col += dims[t]
    return ref, bound
