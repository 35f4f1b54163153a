"""CPU oracle for inverted lists stored as product-quantisation codes.
TEST INFRASTRUCTURE ONLY (tests, smoke check, benchmark baseline); shares no code with
the HIP library.

The paper names product-quantisation codes only as what its on-disk index variant keeps
in memory (Section 6.5 "On-Disk Index": a DiskANN index per partition, whose PQ codes and
cache take a few GB) and fixes no format.  The format here is the build's own reading and
the scoring is the textbook asymmetric computation over such codes, step by step, in
fp64:

  1. The d dimensions are cut into M subspaces of d/M consecutive dimensions.  Subspace m
     has a codebook B[m] of 256 codewords [256, d/M] (float32, given: training a codebook
     is data preparation like training centroids).
  2. A stored vector is M codes c_0 .. c_{M-1}, one byte each, and STANDS FOR the vector
     x^ = B[0][c_0] | B[1][c_1] | ... | B[M-1][c_{M-1}]  (concatenation).
  3. For a query q, the table T[m][c] = <q_m, B[m][c]> for every subspace m and codeword c,
     q_m being the slice of q in subspace m.
  4. score(q, i) = sum over m = 0 .. M-1, in that order, of T[m][code_{i,m}]  ( = <q, x^_i> ).
  5. Probe selection (coarse scores against the fp32 centroids) and the ordering of the
     candidates (score descending, id ascending, position ascending) are those of the flat
     index (oracle/ivf_oracle.py).

The search is exact over the vectors the codes stand for; what the codes lose against the
original embeddings is the caller's trade (tests/test_oracle_pq.py bounds it).

Pins (tests/test_oracle_pq.py): scores equal a library fp64 matmul against the decoded
vectors; all lists probed = exhaustive search over the decoded vectors; codes that
reproduce their vectors exactly reduce to the flat fp32 oracle on those vectors; a
hand-worked case (tests/golden/pq_case.txt); the encoder of the workload generator is a
brute-force nearest codeword and obeys its Cauchy-Schwarz error bound.
"""
from __future__ import annotations

from typing import Tuple

import numpy as np

from . import ivf_oracle as O


def _shape(codes: np.ndarray, codebooks: np.ndarray) -> Tuple[int, int, int]:
    M, ncode, dsub = codebooks.shape
    assert ncode == 256 and codes.dtype == np.uint8 and codes.shape[1] == M
    return M, dsub, M * dsub


def decode(codes: np.ndarray, codebooks: np.ndarray) -> np.ndarray:
    """Step 2: [n, M] codes -> [n, d] float32, each value a copy of a codebook entry."""
    M, dsub, d = _shape(codes, codebooks)
    out = np.empty((codes.shape[0], d), dtype=np.float32)
    for m in range(M):
        out[:, m * dsub:(m + 1) * dsub] = codebooks[m][codes[:, m]]
    return out


def adc_tables(q: np.ndarray, codebooks: np.ndarray) -> np.ndarray:
    """Step 3 for one query: T[m][c] in fp64, each entry a sum over the subspace's
    dimensions in ascending order."""
    M, _, dsub = codebooks.shape
    T = np.zeros((M, 256), dtype=np.float64)
    for m in range(M):
        qm = q[m * dsub:(m + 1) * dsub].astype(np.float64)
        for t in range(dsub):
            T[m] += qm[t] * codebooks[m][:, t].astype(np.float64)
    return T


def adc_scores(T: np.ndarray, codes: np.ndarray) -> np.ndarray:
    """Step 4: scores of the vectors `codes` [n, M] against the query behind T."""
    s = np.zeros(codes.shape[0], dtype=np.float64)
    for m in range(T.shape[0]):
        s += T[m][codes[:, m]]
    return s


def scan_select(codes: np.ndarray, codebooks: np.ndarray, ids: np.ndarray, offsets: np.ndarray,
                Q: np.ndarray, probes: np.ndarray, kout: int) -> Tuple[np.ndarray, np.ndarray]:
    """Steps 3-5 over the probed lists of every query: the first `kout` candidates by
    (score descending, id ascending, position ascending); padding (-1, -inf)."""
    nq = Q.shape[0]
    out_i = np.full((nq, kout), -1, dtype=np.int64)
    out_s = np.full((nq, kout), -np.inf, dtype=np.float64)
    for r in range(nq):
        T = adc_tables(Q[r], codebooks)
        pos = np.concatenate([np.arange(offsets[l], offsets[l + 1]) for l in probes[r]] or
                             [np.empty(0, dtype=np.int64)]).astype(np.int64)
        s = adc_scores(T, codes[pos])
        order = np.lexsort((pos, ids[pos], -s))[:kout]
        out_i[r, :len(order)] = ids[pos[order]]
        out_s[r, :len(order)] = s[order]
    return out_i, out_s


def search(cen: np.ndarray, codes: np.ndarray, codebooks: np.ndarray, ids: np.ndarray,
           offsets: np.ndarray, Q: np.ndarray, nprobe: int, kout: int):
    """(ids[nq,kout], scores[nq,kout] fp64, probes[nq,nprobe], coarse[nq,nlist] fp64)."""
    nprobe = min(int(nprobe), cen.shape[0])
    cs = O.coarse(Q, cen)
    pr = O.probe_select(cs, nprobe)
    oi, os_ = scan_select(codes, codebooks, ids, offsets, Q, pr, kout)
    return oi, os_, pr, cs
