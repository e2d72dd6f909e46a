"""CPU oracle for the multi-LoRA linear layer -- TEST INFRASTRUCTURE ONLY.

Thin ctypes front end over ``multilora_oracle.c`` (naive fp64 loops, one adapter
segment at a time).  Nothing in the product path may import this module; it exists
so that tests, the smoke check and the benchmark's ``cpu_baseline`` leg have an
independent statement of what the layer computes:

    forward   S_i = X_i A_i ;  Y_i = X_i W + s_i S_i B_i          (paper Sec. 2.1, 5.1)
    backward  dS_i = s_i dY_i B_i^T ;  dX_i = dY_i W^T + dS_i A_i^T
              dA_i = X_i^T dS_i ;  dB_i = s_i S_i^T dY_i          (paper Sec. 5.1)

Segments: adapter i owns rows off[i]..off[i+1] of the flattened token buffer
(paper App. A.1, "schedule-driven dispatch": one flat activation buffer, per-adapter
start/end offsets, no padding).  Rows that belong to an adapter of rank 0 are plain
X W rows.

All inputs are float32 numpy arrays that hold exactly the values handed to the GPU
(bf16 inputs are widened, which is exact).  All outputs are float64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "multilora_oracle.c")
_LIB = os.path.join(_HERE, "libmultilora_oracle.so")


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP over the outermost loop only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, dbl, p = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        lib.mlo_num_threads.restype = ctypes.c_int
        lib.mlo_set_num_threads.argtypes = [ctypes.c_int]
        lib.mlo_shrink.argtypes = [i64, i64, i64, p, i64, p, p]
        lib.mlo_fwd_y.argtypes = [i64, p, i64, p, i64, i64, i64, dbl, p, i64, p, p, p, p, p]
        lib.mlo_dshrink.argtypes = [i64, i64, i64, dbl, p, i64, p, p]
        lib.mlo_bwd_dx.argtypes = [i64, p, i64, p, i64, i64, i64, p, i64, p, p, p, p]
        lib.mlo_wgrad_a.argtypes = [i64, i64, i64, i64, p, p, i64, p, p]
        lib.mlo_wgrad_b.argtypes = [i64, i64, i64, dbl, i64, p, p, p, i64, p]
        for f in (lib.mlo_shrink, lib.mlo_fwd_y, lib.mlo_dshrink, lib.mlo_bwd_dx,
                  lib.mlo_wgrad_a, lib.mlo_wgrad_b, lib.mlo_set_num_threads):
            f.restype = None
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().mlo_num_threads())


def set_num_threads(n: int) -> None:
    _load().mlo_set_num_threads(int(n))


def _f32(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.float32:
        raise TypeError("oracle inputs must be float32 arrays holding the exact input values")
    return a


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _idx(ix) -> Optional[np.ndarray]:
    if ix is None:
        return None
    return np.ascontiguousarray(np.asarray(ix, dtype=np.int64))


@dataclass
class Forward:
    """Oracle forward results.  ``Y`` holds the requested rows x columns."""
    Y: np.ndarray                      # [len(rows), len(cols)] float64
    S: List[np.ndarray]                # per adapter [T_i, r_i] float64 (unrounded)
    Ybase: Optional[np.ndarray] = None  # X W alone for the same rows/cols
    rows: Optional[np.ndarray] = None
    cols: Optional[np.ndarray] = None


@dataclass
class Backward:
    dX: np.ndarray                     # [len(rows), len(cols)] float64
    dS: List[np.ndarray]               # per adapter [T_i, r_i]
    dA: List[Optional[np.ndarray]]     # per adapter [k or len(a_rows), r_i]
    dB: List[Optional[np.ndarray]]     # per adapter [r_i, n or len(b_cols)]
    rows: Optional[np.ndarray] = None
    cols: Optional[np.ndarray] = None


def _check_segments(T: int, offsets: Sequence[int]) -> np.ndarray:
    off = np.asarray(offsets, dtype=np.int64)
    if off.ndim != 1 or off.size < 1 or off[0] != 0 or off[-1] != T or np.any(np.diff(off) < 0):
        raise ValueError("segment offsets must start at 0, be non-decreasing and end at T")
    return off


def owner_of_rows(offsets: Sequence[int], rows: np.ndarray) -> np.ndarray:
    """Adapter index that owns each global row (linear definition: off[i] <= t < off[i+1])."""
    off = np.asarray(offsets, dtype=np.int64)
    return (np.searchsorted(off, rows, side="right") - 1).astype(np.int64)


def shrink(X, A, offsets, adapters=None) -> List[Optional[np.ndarray]]:
    """S_i = X_i A_i for every adapter, or only for those listed (others None) (paper Sec. 5.1)."""
    lib = _load()
    X = _f32(X)
    T, k = X.shape
    off = _check_segments(T, offsets)
    out = []
    for i, Ai in enumerate(A):
        if adapters is not None and i not in adapters:
            out.append(None)
            continue
        Ai = _f32(Ai)
        r = Ai.shape[1] if Ai.ndim == 2 else 0
        Ti = int(off[i + 1] - off[i])
        S = np.zeros((Ti, r), dtype=np.float64)
        if Ti and r:
            Xi = X[off[i]:off[i + 1]]
            lib.mlo_shrink(Ti, k, r, _ptr(Xi), k, _ptr(Ai), _ptr(S))
        out.append(S)
    return out


def forward(X, W, A, B, scales, offsets, rows=None, cols=None, want_base=False, adapters=None) -> Forward:
    """Y = X W + s_i (X_i A_i) B_i on the requested global rows / columns (default: all).
    With ``adapters`` given, S_i is computed only for those adapters and for the owners of the
    requested rows (the others are None)."""
    lib = _load()
    X, W = _f32(X), _f32(W)
    T, k = X.shape
    n = W.shape[1]
    assert W.shape[0] == k
    off = _check_segments(T, offsets)
    rows_a = np.arange(T, dtype=np.int64) if rows is None else _idx(rows)
    cols_a = _idx(cols)
    nc = n if cols_a is None else cols_a.size
    own = owner_of_rows(off, rows_a)
    need = None if adapters is None else set(int(a) for a in adapters) | set(int(o) for o in own)
    S = shrink(X, A, off, need)
    Y = np.zeros((rows_a.size, nc), dtype=np.float64)
    Yb = np.zeros_like(Y) if want_base else None
    for i in range(len(A)):
        sel = np.nonzero(own == i)[0]
        if sel.size == 0:
            continue
        Bi = _f32(B[i])
        r = S[i].shape[1]
        local = np.ascontiguousarray(rows_a[sel] - off[i])
        Yi = np.zeros((sel.size, nc), dtype=np.float64)
        Ybi = np.zeros_like(Yi) if want_base else None
        Xi = X[off[i]:off[i + 1]]
        lib.mlo_fwd_y(sel.size, _ptr(local), nc, _ptr(cols_a), k, n, r, float(scales[i]),
                      _ptr(Xi), k, _ptr(W), _ptr(S[i]), _ptr(Bi), _ptr(Yi), _ptr(Ybi))
        Y[sel] = Yi
        if want_base:
            Yb[sel] = Ybi
    return Forward(Y=Y, S=S, Ybase=Yb, rows=rows_a, cols=cols_a)


def backward(dY, X, W, A, B, scales, offsets, S=None, rows=None, cols=None,
             a_rows=None, b_cols=None, adapters=None) -> Backward:
    """dX on the requested rows/cols; dA_i / dB_i for the listed adapters (default all),
    optionally only rows ``a_rows`` of dA_i and columns ``b_cols`` of dB_i; dS_i for all
    adapters, or with ``adapters`` given only for those and for the owners of the requested rows.
    ``S`` defaults to the oracle's own unrounded X_i A_i."""
    lib = _load()
    dY, X, W = _f32(dY), _f32(X), _f32(W)
    T, k = X.shape
    n = W.shape[1]
    off = _check_segments(T, offsets)
    N = len(A)
    rows_a = np.arange(T, dtype=np.int64) if rows is None else _idx(rows)
    own = owner_of_rows(off, rows_a)
    need = None if adapters is None else set(int(a) for a in adapters) | set(int(o) for o in own)
    if S is None:
        S = shrink(X, A, off, need)
    dS = []
    for i in range(N):
        if need is not None and i not in need:
            dS.append(None)
            continue
        Bi = _f32(B[i])
        r = S[i].shape[1]
        Ti = int(off[i + 1] - off[i])
        d = np.zeros((Ti, r), dtype=np.float64)
        if Ti and r:
            lib.mlo_dshrink(Ti, n, r, float(scales[i]), _ptr(dY[off[i]:off[i + 1]]), n, _ptr(Bi), _ptr(d))
        dS.append(d)
    cols_a = _idx(cols)
    nc = k if cols_a is None else cols_a.size
    dX = np.zeros((rows_a.size, nc), dtype=np.float64)
    for i in range(N):
        sel = np.nonzero(own == i)[0]
        if sel.size == 0:
            continue
        Ai = _f32(A[i])
        r = S[i].shape[1]
        local = np.ascontiguousarray(rows_a[sel] - off[i])
        dXi = np.zeros((sel.size, nc), dtype=np.float64)
        lib.mlo_bwd_dx(sel.size, _ptr(local), nc, _ptr(cols_a), k, n, r,
                       _ptr(dY[off[i]:off[i + 1]]), n, _ptr(W), _ptr(dS[i]), _ptr(Ai), _ptr(dXi))
        dX[sel] = dXi
    ar, bc = _idx(a_rows), _idx(b_cols)
    todo = range(N) if adapters is None else list(adapters)
    dA: List[Optional[np.ndarray]] = [None] * N
    dB: List[Optional[np.ndarray]] = [None] * N
    for i in todo:
        r = S[i].shape[1]
        Ti = int(off[i + 1] - off[i])
        na = k if ar is None else ar.size
        nb = n if bc is None else bc.size
        dAi = np.zeros((na, r), dtype=np.float64)
        dBi = np.zeros((r, nb), dtype=np.float64)
        if Ti and r:
            Si = np.ascontiguousarray(S[i], dtype=np.float64)
            lib.mlo_wgrad_a(Ti, k, r, na, _ptr(ar), _ptr(X[off[i]:off[i + 1]]), k, _ptr(dS[i]), _ptr(dAi))
            lib.mlo_wgrad_b(Ti, n, r, float(scales[i]), nb, _ptr(bc), _ptr(Si),
                            _ptr(dY[off[i]:off[i + 1]]), n, _ptr(dBi))
        dA[i], dB[i] = dAi, dBi
    return Backward(dX=dX, dS=dS, dA=dA, dB=dB, rows=rows_a, cols=cols_a)


def flop_count(T, k, n, ranks, seg_lens) -> int:
    """Useful FLOPs of one fwd+bwd: 4Tkn for the two frozen-weight GEMMs and
    6 sum_i T_i r_i (k+n) for shrink, expand, dS, dX_lora, dA, dB (paper Sec. 5.1:
    only the diagonal blocks sum_i T_i r_i are useful work)."""
    r1 = int(sum(int(t) * int(r) for t, r in zip(seg_lens, ranks)))
    return 4 * T * k * n + 6 * r1 * (k + n)
