"""Comparison rules between a search result and the oracle's.  TEST INFRASTRUCTURE
ONLY (tests, smoke check, benchmark baseline); holds no retrieval arithmetic.

Bar (from the benchmark's correctness statement): ids bit-exact, except at positions
where the oracle's adjacent scores differ by less than `tie_rel` relative; scores
within `score_rel` relative, position by position.
"""
from __future__ import annotations

from typing import List, Optional

import numpy as np

TIE_REL = 1e-5
SCORE_REL = {"fp32": 1e-5, "fp16": 2e-3, "int8": 1e-5, "pq8": 1e-5}   # int8, pq8: exact codes, fp32 accumulate
# A score counts as "cancelled" when it is below this fraction of |q|*|x|: its terms have
# eaten at least two decimal digits of each other.  Only such scores may use `abs_floor`.
CANCEL_FRAC = 1e-2


def _near(a: float, b: float, rel: float, floor: float = 0.0) -> bool:
    """|a - b| < rel * max(|a|, |b|); if both are cancelled scores (below CANCEL_FRAC *
    floor), relative to `floor` instead."""
    if a == b:
        return True
    if not (np.isfinite(a) and np.isfinite(b)):
        return False
    m = max(abs(a), abs(b))
    if m < CANCEL_FRAC * floor:
        m = floor
    return abs(a - b) < rel * m


def tie_runs(scores: np.ndarray, rel: float = TIE_REL, floor: float = 0.0) -> List[tuple]:
    """Maximal runs [b, e) of consecutive ranks whose adjacent oracle scores are
    within `rel` of each other."""
    runs, b = [], 0
    for r in range(1, len(scores) + 1):
        if r == len(scores) or not _near(float(scores[r - 1]), float(scores[r]), rel, floor):
            runs.append((b, r))
            b = r
    return runs


def check_topk(got_ids: np.ndarray, got_scores: np.ndarray, ref_ids: np.ndarray,
               ref_scores: np.ndarray, k: int, score_rel: float, tie_rel: float = TIE_REL,
               abs_floor: float = 0.0) -> dict:
    """got_*: [nq, k] from the path under test.  ref_*: [nq, kout >= k+1] from the
    oracle (the extra rows show the gap at the k-th boundary).  Raises
    AssertionError with the first offending query/rank; returns counts.

    `abs_floor` (default 0: purely relative everywhere) is |q|*|x| of the test's data, an
    upper bound of sum|q_t x_t|.  It matters only at ranks whose oracle score has cancelled
    to less than CANCEL_FRAC * abs_floor: an fp32 sum carries an absolute error
    proportional to sum|q_t x_t|, so a score that cancels to ~0 cannot meet a bar relative
    to itself; at those ranks (and for near-tie runs between two such scores) the bars are
    taken relative to abs_floor.  Every other rank gets the pure relative bar.  Tests pass
    it only for unnormalised random data whose results reach down to scores around zero
    (k at or near the candidate count); the configuration tests never do."""
    nq = got_ids.shape[0]
    assert got_ids.shape == (nq, k) and got_scores.shape == (nq, k)
    assert ref_ids.shape[1] >= k + 1, "oracle must supply at least k+1 rows"
    swapped = 0
    for q in range(nq):
        gs = got_scores[q].astype(np.float64)
        rs = ref_scores[q]
        for r in range(k):
            if ref_ids[q, r] < 0:
                assert got_ids[q, r] == -1 and np.isneginf(gs[r]), \
                    f"q{q} rank{r}: expected padding (-1,-inf), got ({got_ids[q, r]},{gs[r]})"
                continue
            mag = abs(rs[r]) if abs(rs[r]) >= CANCEL_FRAC * abs_floor else abs_floor
            tol = score_rel * max(mag, 1e-30)
            assert abs(gs[r] - rs[r]) <= tol, \
                f"q{q} rank{r}: score {gs[r]!r} vs oracle {rs[r]!r} (tol {tol:.3g})"
        assert np.all(gs[:-1] >= gs[1:]), f"q{q}: scores not non-increasing"
        real = got_ids[q][got_ids[q] >= 0]
        assert len(np.unique(real)) == len(real), f"q{q}: duplicate ids"
        valid = int((ref_ids[q] >= 0).sum())
        for b, e in tie_runs(rs[:valid], tie_rel, abs_floor):
            if b >= k:
                break
            ee = min(e, k)
            want = set(int(x) for x in ref_ids[q, b:e])
            got = [int(x) for x in got_ids[q, b:ee]]
            if e > k or e - b > 1:
                if e == ref_ids.shape[1] and e > k:
                    raise AssertionError(f"q{q}: near-tie run reaches past the oracle's {e} rows; "
                                         "ask the oracle for more rows")
                assert set(got) <= want and len(set(got)) == len(got), \
                    f"q{q} ranks[{b},{ee}): ids {got} not within tied oracle ids {sorted(want)}"
                if got != [int(x) for x in ref_ids[q, b:ee]]:
                    swapped += 1
            else:
                assert got[0] == int(ref_ids[q, b]), \
                    f"q{q} rank{b}: id {got[0]} vs oracle {int(ref_ids[q, b])} " \
                    f"(scores {gs[b]!r} / {rs[b]!r})"
    return {"queries": nq, "tie_runs_reordered": swapped}


def check_probes(got_probes: np.ndarray, coarse: np.ndarray, nprobe: int,
                 tie_rel: float = TIE_REL) -> bool:
    """got_probes [nq, nprobe] (any order) against the oracle's fp64 coarse scores.
    A list may replace another only if both lie within `tie_rel` of the score at the
    nprobe-th boundary.  Returns True iff the probe SETS are identical to the
    oracle's (then no re-run of the scan on the reported probes is needed)."""
    nq, nlist = coarse.shape
    same = True
    for q in range(nq):
        order = np.lexsort((np.arange(nlist), -coarse[q]))
        ref = set(int(x) for x in order[:nprobe])
        got = [int(x) for x in got_probes[q]]
        assert len(set(got)) == nprobe and all(0 <= g < nlist for g in got), \
            f"q{q}: probe list has duplicates or out-of-range entries"
        if set(got) == ref:
            continue
        same = False
        edge = float(coarse[q, order[nprobe - 1]])
        for l in set(got) ^ ref:
            assert _near(float(coarse[q, l]), edge, tie_rel), \
                f"q{q}: list {l} (coarse {coarse[q, l]!r}) differs from the oracle's probe set " \
                f"and is not a near-tie of the boundary score {edge!r}"
    return same


def check_ids_in_probed_lists(got_ids: np.ndarray, probes: np.ndarray, ids: np.ndarray,
                              offsets: np.ndarray) -> None:
    """Every returned id belongs to a list the query probed."""
    for q in range(got_ids.shape[0]):
        allowed = np.concatenate([ids[offsets[l]:offsets[l + 1]] for l in probes[q]] or [np.empty(0, np.int64)])
        real = got_ids[q][got_ids[q] >= 0]
        assert np.isin(real, allowed).all(), f"q{q}: an id lies outside the probed lists"
