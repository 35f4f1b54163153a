"""ctypes front of the plain-C CPU oracle (oracle/ivf_oracle.c).

TEST INFRASTRUCTURE ONLY.  The product path never imports this module; it is used
by tests/, by the smoke check and by the benchmark's cpu_baseline leg.  It shares
no code with the HIP library.  The arithmetic lives in the C file; this module only
marshals NumPy arrays and composes the three steps in the order the definition
gives them (coarse scores -> probe lists -> scan and sorted selection).

Pins (see tests/test_oracle_*.py): exhaustive equality with a library fp64 matmul +
sort when nprobe = nlist, a library brute-force L2 k-NN on normalised data, a
hand-written closed-form case (tests/golden/basis_case.txt), the half-precision
decoder against NumPy for all 65536 bit patterns, ordering/uniqueness/probe-set
invariants, prefix and merge properties of the selection, and monotonicity in nprobe.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ivf_oracle.c")
_LIB = os.path.join(_HERE, "libivf_oracle.so")


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP, no fast-math: every sum keeps its
    written order)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oracle_half_to_double.restype = C.c_double
        _lib.oracle_half_to_double.argtypes = [C.c_uint16]
        _lib.oracle_threads.restype = C.c_int
        for name in ("oracle_coarse", "oracle_probe_select", "oracle_scan_select", "oracle_assign"):
            getattr(_lib, name).restype = C.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _vec(x: np.ndarray) -> Tuple[np.ndarray, int]:
    if x.dtype == np.float32:
        return np.ascontiguousarray(x), 0
    if x.dtype == np.float16:
        return np.ascontiguousarray(x), 1
    if x.dtype == np.uint8:          # int8 storage: records of d codes + fp32 scale
        return np.ascontiguousarray(x), 2
    raise TypeError("vectors must be float32, float16 or uint8 records (int8 codes + fp32 scale)")


def _dim(X: np.ndarray, dt: int) -> int:
    return X.shape[1] - 4 if dt == 2 else X.shape[1]


def threads() -> int:
    return int(lib().oracle_threads())


def half_to_double(bits: int) -> float:
    return float(lib().oracle_half_to_double(C.c_uint16(bits)))


def coarse(Q: np.ndarray, cen: np.ndarray) -> np.ndarray:
    Q = np.ascontiguousarray(Q, dtype=np.float32)
    cen = np.ascontiguousarray(cen, dtype=np.float32)
    nq, d = Q.shape
    nlist = cen.shape[0]
    assert cen.shape[1] == d
    out = np.empty((nq, nlist), dtype=np.float64)
    rc = lib().oracle_coarse(_p(Q), C.c_int64(nq), _p(cen), C.c_int64(nlist), C.c_int(d), _p(out))
    assert rc == 0, rc
    return out


def probe_select(coarse_scores: np.ndarray, nprobe: int) -> np.ndarray:
    cs = np.ascontiguousarray(coarse_scores, dtype=np.float64)
    nq, nlist = cs.shape
    out = np.empty((nq, nprobe), dtype=np.int32)
    rc = lib().oracle_probe_select(_p(cs), C.c_int64(nq), C.c_int64(nlist), C.c_int(nprobe), _p(out))
    assert rc == 0, rc
    return out


def scan_select(vectors: np.ndarray, ids: np.ndarray, offsets: np.ndarray, Q: np.ndarray,
                probes: np.ndarray, kout: int) -> Tuple[np.ndarray, np.ndarray]:
    X, dt = _vec(vectors)
    ids = np.ascontiguousarray(ids, dtype=np.int64)
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    Q = np.ascontiguousarray(Q, dtype=np.float32)
    probes = np.ascontiguousarray(probes, dtype=np.int32)
    nq, d = Q.shape
    assert _dim(X, dt) == d and probes.shape[0] == nq
    nlist = offsets.shape[0] - 1
    out_ids = np.empty((nq, kout), dtype=np.int64)
    out_s = np.empty((nq, kout), dtype=np.float64)
    rc = lib().oracle_scan_select(_p(X), C.c_int(dt), _p(ids), _p(offsets), C.c_int64(nlist),
                                  C.c_int(d), _p(Q), C.c_int64(nq), _p(probes),
                                  C.c_int(probes.shape[1]), C.c_int(kout), _p(out_ids), _p(out_s))
    assert rc == 0, rc
    return out_ids, out_s


def search(cen: np.ndarray, vectors: np.ndarray, ids: np.ndarray, offsets: np.ndarray,
           Q: np.ndarray, nprobe: int, kout: int):
    """The whole definition: returns (ids[nq,kout], scores[nq,kout] fp64,
    probes[nq,nprobe], coarse[nq,nlist] fp64).  Callers that check a top-k ask for
    kout = k+1 so the gap at the k-th boundary is visible.  nprobe above nlist
    means every list."""
    nprobe = min(int(nprobe), cen.shape[0])
    cs = coarse(Q, cen)
    pr = probe_select(cs, nprobe)
    oi, os_ = scan_select(vectors, ids, offsets, Q, pr, kout)
    return oi, os_, pr, cs


def assign(vectors: np.ndarray, cen: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    X, dt = _vec(vectors)
    cen = np.ascontiguousarray(cen, dtype=np.float32)
    n, d = X.shape
    out = np.empty(n, dtype=np.int32)
    best = np.empty(n, dtype=np.float64)
    rc = lib().oracle_assign(_p(X), C.c_int(dt), C.c_int64(n), _p(cen), C.c_int64(cen.shape[0]),
                             C.c_int(d), _p(out), _p(best))
    assert rc == 0, rc
    return out, best
