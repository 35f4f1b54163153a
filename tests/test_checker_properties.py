"""Randomised properties of the comparison rules (oracle/check.py) that every parity claim
rests on: a result that differs from the oracle's only by reordering ids inside near-tie
runs, with scores within the bar, is accepted; any id moved across a real gap, any id from
outside, any score off by more than the bar, any duplicate or missing padding is rejected."""
import numpy as np
import pytest

from oracle import check as CK


def _oracle_rows(rng, k, extra, ties):
    """Strictly decreasing oracle scores with a few planted near-tie runs; unique ids."""
    n = k + extra
    gaps = rng.uniform(2e-3, 5e-2, size=n)
    runs = []
    for _ in range(ties):
        b = int(rng.integers(0, n - 1))
        e = min(n, b + int(rng.integers(2, 5)))
        gaps[b + 1:e] = rng.uniform(1e-9, 2e-7, size=e - b - 1)      # far inside the 1e-5 relative bar
        runs.append((b, e))
    scores = 10.0 - np.cumsum(gaps)
    ids = rng.permutation(10 * n)[:n].astype(np.int64)
    return ids[None, :], scores[None, :], runs


@pytest.mark.parametrize("seed", range(30))
def test_permutations_inside_near_tie_runs_are_accepted_and_nothing_else(seed):
    rng = np.random.default_rng(seed)
    k = int(rng.integers(3, 25))
    ref_ids, ref_s, _ = _oracle_rows(rng, k, extra=6, ties=int(rng.integers(0, 4)))
    runs = CK.tie_runs(ref_s[0])
    # a legal result: shuffle ids inside every run, keep scores (within 1e-6 relative)
    got_full = ref_ids[0].copy()
    for b, e in runs:
        got_full[b:e] = rng.permutation(got_full[b:e])
    got_ids = got_full[:k][None, :].copy()
    got_s = (ref_s[0, :k] * (1 + rng.uniform(-1e-6, 1e-6, size=k))).astype(np.float32)
    got_s = np.sort(got_s)[::-1][None, :].copy()
    res = CK.check_topk(got_ids, got_s, ref_ids, ref_s, k, 1e-5)
    assert res["queries"] == 1

    def rejected(ids, scores):
        with pytest.raises(AssertionError):
            CK.check_topk(ids, scores, ref_ids, ref_s, k, 1e-5)

    # an id moved across a real gap
    for b, e in runs:
        if e < k and b < e:                      # swap the last of this run with the first of the next
            bad = ref_ids[0, :k][None, :].copy()
            bad[0, e - 1], bad[0, e] = bad[0, e], bad[0, e - 1]
            rejected(bad, got_s)
            break
    # an id that the oracle does not have at all
    bad = got_ids.copy()
    bad[0, int(rng.integers(0, k))] = 10**9
    rejected(bad, got_s)
    # a duplicate
    if k >= 2:
        bad = got_ids.copy()
        bad[0, 1] = bad[0, 0]
        rejected(bad, got_s)
    # a score off by ten times the bar
    bad_s = got_s.copy()
    j = int(rng.integers(0, k))
    bad_s[0, j] = np.float32(bad_s[0, j] * (1 + 1e-4))
    rejected(got_ids, bad_s)
    # scores out of order
    if k >= 2 and got_s[0, 0] != got_s[0, -1]:
        rejected(got_ids, got_s[:, ::-1].copy())


def test_padding_is_required_exactly_where_the_oracle_pads():
    ref_ids = np.array([[5, 9, -1, -1, -1]], dtype=np.int64)
    ref_s = np.array([[2.0, 1.0, -np.inf, -np.inf, -np.inf]])
    ok_ids = np.array([[5, 9, -1, -1]], dtype=np.int64)
    ok_s = np.array([[2.0, 1.0, -np.inf, -np.inf]], dtype=np.float32)
    CK.check_topk(ok_ids, ok_s, ref_ids, ref_s, 4, 1e-5)
    for bad_ids, bad_s in ((np.array([[5, 9, 0, -1]]), ok_s), (ok_ids, np.array([[2.0, 1.0, 0.0, -np.inf]], dtype=np.float32)),
                           (np.array([[5, -1, -1, -1]]), np.array([[2.0, -np.inf, -np.inf, -np.inf]], dtype=np.float32))):
        with pytest.raises(AssertionError):
            CK.check_topk(bad_ids.astype(np.int64), bad_s, ref_ids, ref_s, 4, 1e-5)


def test_a_tie_run_that_reaches_past_the_oracle_rows_asks_for_more_rows():
    ref_ids = np.array([[1, 2, 3, 4]], dtype=np.int64)
    ref_s = np.array([[1.0, 0.5, 0.5 - 1e-9, 0.5 - 2e-9]])          # the run [1, 4) touches the last oracle row
    got_ids = np.array([[1, 3, 2]], dtype=np.int64)
    got_s = np.array([[1.0, 0.5, 0.5]], dtype=np.float32)
    with pytest.raises(AssertionError, match="more rows"):
        CK.check_topk(got_ids, got_s, ref_ids, ref_s, 3, 1e-5)


@pytest.mark.parametrize("seed", range(10))
def test_probe_sets_may_differ_only_at_a_near_tied_boundary(seed):
    rng = np.random.default_rng(100 + seed)
    nlist, nprobe = 40, 6
    coarse = np.sort(rng.uniform(0.2, 1.0, size=nlist))[::-1][None, :].copy()
    coarse[0] = coarse[0][rng.permutation(nlist)]
    order = np.lexsort((np.arange(nlist), -coarse[0]))
    ref = order[:nprobe].astype(np.int32)[None, :]
    assert CK.check_probes(ref[:, ::-1].copy(), coarse, nprobe) is True          # order inside the set is free
    # the next list in line is not a near-tie: not accepted
    bad = ref.copy()
    bad[0, -1] = order[nprobe]
    with pytest.raises(AssertionError):
        CK.check_probes(bad, coarse, nprobe)
    # make it a near-tie of the boundary: accepted, and reported as a different set
    c2 = coarse.copy()
    c2[0, order[nprobe]] = c2[0, order[nprobe - 1]] * (1 - 1e-7)
    assert CK.check_probes(bad, c2, nprobe) is False
    # duplicates and out-of-range entries are never accepted
    dup = ref.copy()
    dup[0, 0] = dup[0, 1]
    with pytest.raises(AssertionError):
        CK.check_probes(dup, coarse, nprobe)


def test_abs_floor_only_loosens_ranks_whose_score_has_cancelled():
    """With a floor of |q||x| = 100 the ranks at 40 and 3 keep the pure 1e-5 relative bar;
    only the ranks below 1 % of the floor (0.02, -0.01) are compared relative to the floor."""
    ref_ids = np.array([[1, 2, 3, 4, 5]], dtype=np.int64)
    ref_s = np.array([[40.0, 3.0, 0.02, -0.01, -7.0]])
    ids = ref_ids[:, :4].copy()
    exact = ref_s[:, :4].astype(np.float32)
    CK.check_topk(ids, exact, ref_ids, ref_s, 4, 1e-5, abs_floor=100.0)
    # a cancelled score off by 5e-4 absolute: within 1e-5 * 100, far outside 1e-5 * 0.02
    off = exact.copy()
    off[0, 2] += np.float32(5e-4)
    CK.check_topk(ids, off, ref_ids, ref_s, 4, 1e-5, abs_floor=100.0)
    with pytest.raises(AssertionError):
        CK.check_topk(ids, off, ref_ids, ref_s, 4, 1e-5)
    # the same absolute error on a score that has not cancelled is rejected, floor or not
    off = exact.copy()
    off[0, 1] += np.float32(5e-4)
    with pytest.raises(AssertionError):
        CK.check_topk(ids, off, ref_ids, ref_s, 4, 1e-5, abs_floor=100.0)
    # ids: two cancelled scores 1e-4 apart may swap under the floor, 3.0 and 3.0001 may not
    swapped = ids.copy()
    swapped[0, 2], swapped[0, 3] = ids[0, 3], ids[0, 2]
    near = ref_s.copy()
    near[0, 3] = 0.02 - 1e-4
    got = near[:, :4].astype(np.float32)
    CK.check_topk(swapped, got, ref_ids, near, 4, 1e-5, abs_floor=100.0)
    with pytest.raises(AssertionError):
        CK.check_topk(swapped, got, ref_ids, near, 4, 1e-5)
    near = ref_s.copy()
    near[0, 1] = 3.0
    near[0, 2] = 3.0 - 1e-4
    swapped = ids.copy()
    swapped[0, 1], swapped[0, 2] = ids[0, 2], ids[0, 1]
    with pytest.raises(AssertionError):
        CK.check_topk(swapped, near[:, :4].astype(np.float32), ref_ids, near, 4, 1e-5, abs_floor=100.0)
