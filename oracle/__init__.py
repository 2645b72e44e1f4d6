"""CPU oracle for RSR matrix-vector multiplication (test infrastructure only).

Thin ctypes wrapper around ``rsr_oracle.c`` (plain C, float64).  Nothing in
the product imports this package; only ``tests/``, ``__graft_entry__.smoke()``
and the ``cpu_baseline`` leg of ``bench.py`` do.  It shares no code with the
HIP library.  The arithmetic lives in the C file; this module only marshals
numpy arrays and strings the per-block steps together in the order the paper
gives them (System Overview: preprocess = split into k-row blocks, group
identical column patterns; inference = aggregate per group, then distribute
once per group).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import List

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rsr_oracle.c")
_LIB = os.path.join(_HERE, "librsr_oracle.so")

BINARY = 0
TERNARY_2PASS = 1
TERNARY_FUSED = 2

MODE_BINARY, MODE_POS, MODE_NEG, MODE_FUSED3 = 0, 1, 2, 3


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no optimisation tricks, -O2 only)."""
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < os.path.getmtime(_SRC))
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared",
                               "-Wall", "-Wextra", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, dbl, vp = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        lib.rsr_oracle_num_patterns.restype = i64
        lib.rsr_oracle_num_patterns.argtypes = [ctypes.c_int, ctypes.c_int]
        lib.rsr_oracle_dense.argtypes = [vp, i64, i64, vp, dbl, vp]
        lib.rsr_oracle_encode.argtypes = [vp, i64, i64, ctypes.c_int, ctypes.c_int, vp]
        lib.rsr_oracle_sort.argtypes = [vp, i64, i64, i64, vp, vp]
        lib.rsr_oracle_segment_sums.restype = None
        lib.rsr_oracle_segment_sums.argtypes = [vp, vp, i64, vp, vp]
        lib.rsr_oracle_expand.restype = None
        lib.rsr_oracle_expand.argtypes = [vp, i64, ctypes.c_int, ctypes.c_int, vp]
        lib.rsr_oracle_matvec_pass.argtypes = [vp, vp, i64, i64, ctypes.c_int,
                                               ctypes.c_int, vp, dbl, ctypes.c_int, vp]
        lib.rsr_oracle_pack2.argtypes = [vp, i64, i64, i64, vp]
        lib.rsr_oracle_unpack2.argtypes = [vp, i64, i64, i64, vp]
        _lib = lib
    return _lib


def _p(a: np.ndarray) -> int:
    return a.ctypes.data


def _as_m(M) -> np.ndarray:
    M = np.ascontiguousarray(M, dtype=np.int8)
    if M.ndim != 2:
        raise ValueError("M must be 2-D")
    return M


def num_patterns(k: int, mode: int) -> int:
    return int(_load().rsr_oracle_num_patterns(k, mode))


def dense_matvec(M, v, scale: float = 1.0) -> np.ndarray:
    """out = scale * M v by the definition, float64."""
    M = _as_m(M)
    v = np.ascontiguousarray(v, dtype=np.float64)
    if v.shape != (M.shape[1],):
        raise ValueError("v has the wrong length")
    out = np.empty(M.shape[0], dtype=np.float64)
    _load().rsr_oracle_dense(_p(M), M.shape[0], M.shape[1], _p(v), float(scale), _p(out))
    return out


def encode(M, k: int, mode: int) -> np.ndarray:
    """Pattern code of every (block, column): uint32 [nb][cols]."""
    M = _as_m(M)
    rows, cols = M.shape
    nb = (rows + k - 1) // k
    code = np.empty((nb, cols), dtype=np.uint32)
    rc = _load().rsr_oracle_encode(_p(M), rows, cols, k, mode, _p(code))
    if rc:
        raise ValueError("matrix entry outside the alphabet of mode %d" % mode)
    return code


def counting_sort(code: np.ndarray, P: int):
    """Stable counting sort per block -> (pi [nb][cols], off [nb][P+1])."""
    code = np.ascontiguousarray(code, dtype=np.uint32)
    nb, cols = code.shape
    pi = np.empty((nb, cols), dtype=np.uint32)
    off = np.empty((nb, P + 1), dtype=np.uint32)
    rc = _load().rsr_oracle_sort(_p(code), nb, cols, P, _p(pi), _p(off))
    if rc:
        raise MemoryError
    return pi, off


def segment_sums(pi_b, off_b, v) -> np.ndarray:
    pi_b = np.ascontiguousarray(pi_b, dtype=np.uint32)
    off_b = np.ascontiguousarray(off_b, dtype=np.uint32)
    v = np.ascontiguousarray(v, dtype=np.float64)
    P = off_b.shape[0] - 1
    u = np.empty(P, dtype=np.float64)
    _load().rsr_oracle_segment_sums(_p(pi_b), _p(off_b), P, _p(v), _p(u))
    return u


def expand(u, k: int, mode: int) -> np.ndarray:
    """y = u * B_k for one block (k outputs)."""
    u = np.ascontiguousarray(u, dtype=np.float64)
    y = np.empty(k, dtype=np.float64)
    _load().rsr_oracle_expand(_p(u), u.shape[0], k, mode, _p(y))
    return y


@dataclass
class Pass:
    mode: int
    sign: float
    pi: np.ndarray    # uint32 [nb][cols]
    off: np.ndarray   # uint32 [nb][P+1]


@dataclass
class Artifacts:
    rows: int
    cols: int
    k: int
    kind: int
    passes: List[Pass]


def preprocess(M, k: int, kind: int) -> Artifacts:
    """Offline phase: per block, encode, counting-sort, emit boundaries."""
    M = _as_m(M)
    rows, cols = M.shape
    if kind == BINARY:
        plan = [(MODE_BINARY, 1.0)]
    elif kind == TERNARY_2PASS:
        plan = [(MODE_POS, 1.0), (MODE_NEG, -1.0)]
    elif kind == TERNARY_FUSED:
        plan = [(MODE_FUSED3, 1.0)]
    else:
        raise ValueError("unknown kind")
    passes = []
    for mode, sign in plan:
        code = encode(M, k, mode)
        pi, off = counting_sort(code, num_patterns(k, mode))
        passes.append(Pass(mode, sign, pi, off))
    return Artifacts(rows, cols, k, kind, passes)


def matvec(art: Artifacts, v, scale: float = 1.0) -> np.ndarray:
    """Online phase: aggregate per group, distribute once per group."""
    v = np.ascontiguousarray(v, dtype=np.float64)
    if v.shape != (art.cols,):
        raise ValueError("v has the wrong length")
    out = np.zeros(art.rows, dtype=np.float64)
    for n, p in enumerate(art.passes):
        rc = _load().rsr_oracle_matvec_pass(_p(p.pi), _p(p.off), art.rows, art.cols,
                                            art.k, p.mode, _p(v), p.sign * float(scale),
                                            1 if n else 0, _p(out))
        if rc:
            raise MemoryError
    return out


def pack2(M) -> np.ndarray:
    """Dense 2-bit packing of a ternary matrix: uint8 [rows][ceil(cols/4)]."""
    M = _as_m(M)
    rows, cols = M.shape
    rb = (cols + 3) // 4
    packed = np.empty((rows, rb), dtype=np.uint8)
    rc = _load().rsr_oracle_pack2(_p(M), rows, cols, rb, _p(packed))
    if rc:
        raise ValueError("not a ternary matrix")
    return packed


def unpack2(packed, cols: int) -> np.ndarray:
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    rows, rb = packed.shape
    M = np.empty((rows, cols), dtype=np.int8)
    rc = _load().rsr_oracle_unpack2(_p(packed), rows, cols, rb, _p(M))
    if rc:
        raise ValueError("unused 2-bit symbol in packed data")
    return M
