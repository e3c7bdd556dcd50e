"""ctypes wrapper of contract_plain.c: the literal ascending-k fp32 contraction (oracle pin; test infrastructure only).

`build()` compiles it with gcc next to this file; `contract_nt(x, w)` returns x @ w.T with one fp32 accumulator per
output element taking the products in ascending k (Section 3.1: operands in half precision, sums in single)."""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "contract_plain.c")
LIB = os.path.join(HERE, "liboracle_contract.so")


def build() -> str:
    cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC", "-o", LIB, SRC]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"gcc failed for {SRC}:\n{r.stdout}\n{r.stderr}")
    return LIB


_lib = None


def contract_nt(x: np.ndarray, w: np.ndarray) -> np.ndarray:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
            build()
        _lib = ctypes.CDLL(LIB)
        _lib.oracle_contract_nt_f32.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_long] * 3
        _lib.oracle_contract_nt_f32.restype = None
    x = np.ascontiguousarray(x, dtype=np.float32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    assert x.ndim == 2 and w.ndim == 2 and x.shape[1] == w.shape[1]
    y = np.empty((x.shape[0], w.shape[0]), dtype=np.float32)
    _lib.oracle_contract_nt_f32(x.ctypes.data, w.ctypes.data, y.ctypes.data, x.shape[0], w.shape[0], x.shape[1])
    return y
