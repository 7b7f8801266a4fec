"""CPU ORACLE -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT.

Python face of `lora_oracle.c` (the fp64 definition of the batched
heterogeneous-rank LoRA apply, paper section 3.1) and of `indexer.py` (the
integer work lists).  `manager.py` (cache manager, section 4.2) and
`scheduler.py` (request scheduler, section 4.3) are imported by their tests
directly.  Only `tests/`, `__graft_entry__.smoke()` and the
`cpu_baseline` leg of `bench.py` import this package.  It imports nothing from
the GPU package and shares no code with it.

Pins (tests/test_oracle_pins.py): a hand-worked example, per-token dense
W + s.A.B brute force through numpy's matmul, the single-adapter batch as one
GEMM, identity-slice and one-hot closed forms, and the invariants (zero B,
zero scale, linearity in x, segment permutation, segment splitting, zero-padded
rank growth, additivity of two adapters).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, Sequence, Tuple

import numpy as np

from .indexer import index, token_map  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lora_oracle.c")
_LIB = os.path.join(_HERE, "liblora_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, OpenMP over tokens)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", _SRC, "-o", _LIB])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        lib.oracle_lora_apply.restype = ctypes.c_int
        lib.oracle_lora_apply.argtypes = [
            ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, dp, dp, dp, ctypes.c_int32, ip, ip,
            ctypes.c_int32, ip, ctypes.POINTER(dp), ctypes.POINTER(dp), dp, ctypes.c_double,
        ]
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def lora_apply(
    x: np.ndarray,
    base: np.ndarray,
    seg_offsets: Sequence[int],
    seg_adapter: Sequence[int],
    adapters: Dict[int, Tuple[np.ndarray, np.ndarray, float]],
    scale: float,
) -> np.ndarray:
    """y[t] = base[t] + scale*alpha_i * (x[t] @ A_i) @ B_i, in fp64, for every token t of
    a segment whose adapter index i is >= 0; other tokens keep base[t].

    `adapters` maps an adapter index to (A [h_in][r], B [r][h_out], alpha).  Inputs of any
    float dtype are widened to double exactly.
    """
    lib = _load()
    x = np.ascontiguousarray(x, np.float64)
    base = np.ascontiguousarray(base, np.float64)
    T, h_in = x.shape
    h_out = base.shape[1]
    assert base.shape[0] == T
    so = np.ascontiguousarray(seg_offsets, np.int32)
    sa = np.ascontiguousarray(seg_adapter, np.int32)
    n_ad = (max(adapters) + 1) if adapters else 0
    n_ad = max(n_ad, int(sa.max()) + 1 if len(sa) else 0, 1)
    rank = np.zeros(n_ad, np.int32)
    alpha = np.ones(n_ad, np.float64)
    dp = ctypes.POINTER(ctypes.c_double)
    Ap = (dp * n_ad)()
    Bp = (dp * n_ad)()
    keep = []
    lens = np.diff(so) if len(so) == len(sa) + 1 else np.zeros(len(sa), np.int64)
    for i in set(int(v) for v, n in zip(sa, lens) if v >= 0 and n > 0):  # empty segments need no weights
        if i not in adapters:
            raise KeyError(f"segment names adapter {i} which was not supplied")
    for i, (A, B, al) in adapters.items():
        A = np.ascontiguousarray(A, np.float64)
        B = np.ascontiguousarray(B, np.float64)
        assert A.shape[0] == h_in and B.shape[1] == h_out and A.shape[1] == B.shape[0]
        rank[i] = A.shape[1]
        alpha[i] = float(al)
        keep += [A, B]
        Ap[i] = A.ctypes.data_as(dp)
        Bp[i] = B.ctypes.data_as(dp)
    y = np.empty((T, h_out), np.float64)
    ip = ctypes.POINTER(ctypes.c_int32)
    rc = lib.oracle_lora_apply(
        T, h_in, h_out, x.ctypes.data_as(dp), base.ctypes.data_as(dp), y.ctypes.data_as(dp), len(sa),
        so.ctypes.data_as(ip), sa.ctypes.data_as(ip), n_ad, rank.ctypes.data_as(ip), Ap, Bp,
        alpha.ctypes.data_as(dp), float(scale),
    )
    if rc != 0:
        raise ValueError(f"oracle_lora_apply rejected its input (code {rc})")
    return y
