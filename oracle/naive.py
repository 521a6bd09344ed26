"""ctypes access to the naive C oracle (forward_naive.c) -- TEST INFRASTRUCTURE ONLY.

build() compiles it with gcc into oracle/_build/; load() returns the library and
fails loudly if it has not been built.  The wrappers take the same unit
dictionaries as glowq_oracle.py (numpy arrays of bit patterns).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "forward_naive.c")
_LIB = os.path.join(_HERE, "_build", "libglowq_oracle.so")
_ACT = {"f16": 0, "bf16": 1}
_lib = None


def build(force: bool = True) -> str:
    os.makedirs(os.path.dirname(_LIB), exist_ok=True)
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build(force=False)
        _lib = ctypes.CDLL(_LIB)
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def max_threads() -> int:
    return int(load().glowq_oracle_max_threads())


def unpack(wq: np.ndarray) -> np.ndarray:
    wq = np.ascontiguousarray(wq, np.uint32)
    O, n = wq.shape
    q = np.empty((O, n * 8), np.uint8)
    rc = load().glowq_oracle_unpack(_p(wq), O, n * 8, _p(q))
    assert rc == 0
    return q


def dequant(module: dict, G: int, act: str) -> np.ndarray:
    wq = np.ascontiguousarray(module["wq"], np.uint32)
    s = np.ascontiguousarray(module["scales"], np.uint16)
    z = np.ascontiguousarray(module["zeros"], np.uint16)
    O, n = wq.shape
    out = np.empty((O, n * 8), np.float64)
    rc = load().glowq_oracle_dequant(_p(wq), _p(s), _p(z), O, n * 8, G, _ACT[act], _p(out))
    assert rc == 0
    return out


def shared_proj(X_bits: np.ndarray, B_bits: np.ndarray, act: str) -> np.ndarray:
    X = np.ascontiguousarray(X_bits, np.uint16)
    B = np.ascontiguousarray(B_bits, np.uint16)
    T, d = X.shape
    r = B.shape[0]
    R = np.empty((T, r), np.float64)
    rc = load().glowq_oracle_shared_proj(_p(X), _p(B), T, d, r, _ACT[act], _p(R))
    assert rc == 0
    return R


def module_forward(module: dict, X_bits: np.ndarray, R: Optional[np.ndarray], G: int,
                   act: str, rows: Optional[np.ndarray] = None) -> np.ndarray:
    """Y[T][n_rows] float64; `rows` picks output rows (None = all)."""
    wq = np.ascontiguousarray(module["wq"], np.uint32)
    s = np.ascontiguousarray(module["scales"], np.uint16)
    z = np.ascontiguousarray(module["zeros"], np.uint16)
    X = np.ascontiguousarray(X_bits, np.uint16)
    T, d = X.shape
    O = wq.shape[0]
    A = Rc = None
    r = 0
    if R is not None:
        A = np.ascontiguousarray(module["A"], np.uint16)
        Rc = np.ascontiguousarray(R, np.float64)
        r = A.shape[1]
        assert Rc.shape == (T, r)
    if rows is not None:
        rows = np.ascontiguousarray(rows, np.int32)
        assert rows.min(initial=0) >= 0 and rows.max(initial=0) < O
    n_rows = O if rows is None else rows.shape[0]
    Y = np.empty((T, n_rows), np.float64)
    rc = load().glowq_oracle_module_forward(_p(wq), _p(s), _p(z), _p(A), _p(X), _p(Rc), T, d,
                                            O, r, G, _ACT[act], _p(rows), n_rows, _p(Y))
    assert rc == 0
    return Y


def group_forward(unit: dict, restore: bool = True,
                  rows: Optional[Sequence[Optional[np.ndarray]]] = None) -> List[np.ndarray]:
    act, G = unit["act"], unit["G"]
    R = None
    if restore and unit["r"] > 0:
        R = shared_proj(unit["X"], unit["B"], act)
    out = []
    for i, m in enumerate(unit["modules"]):
        out.append(module_forward(m, unit["X"], R, G, act, None if rows is None else rows[i]))
    return out


if __name__ == "__main__":
    print(build())
