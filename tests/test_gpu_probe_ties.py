"""GPU probe selection at the nprobe-th boundary: exact duplicate centroids inside, at and
just past the boundary (ties go to the smaller list number), centroids whose coarse
scores fp32 cannot tell apart although fp64 can (the GPU's probe set then differs from
the oracle's by a near-tie, and the oracle re-scans the GPU's set), and centroids within
1e-6 relative of the boundary score.  Coarse scores are <q, centroid>; the benchmark's
mixture data never comes near such ties, so these are hand-made."""
import numpy as np
import pytest

from oracle import check as CK
from oracle import ivf_oracle as O
from paper_2504_15302_amd import ivf
from tests.gpu_util import check_against_oracle, gpu_search, say

pytestmark = pytest.mark.gpu


def _graded_index(nlist, d, alphas, seed, per_list=70, storage=np.float32, extra_dim=None):
    """Centroid j = alphas[j] * u (+ an optional component on a second axis), so that the
    coarse score of the query u is alphas[j]: the caller decides the order and the ties.
    Every list holds `per_list` random vectors with distinct content."""
    rng = np.random.default_rng(seed)
    u = np.zeros(d, dtype=np.float32)
    u[0] = 1.0
    cen = np.zeros((nlist, d), dtype=np.float32)
    cen[:, 0] = np.asarray(alphas, dtype=np.float32)
    if extra_dim is not None:
        for j, v in extra_dim.items():
            cen[j, 1] = np.float32(v)
    n = nlist * per_list
    vec = rng.standard_normal((n, d)).astype(storage)
    ids = rng.permutation(3 * n)[:n].astype(np.int64)
    off = np.arange(0, n + 1, per_list, dtype=np.int64)
    return cen, np.ascontiguousarray(vec), ids, off, u


def _run(cen, vec, ids, off, q, nprobe, k, storage="fp32"):
    idx = ivf.Index()
    idx.upload(cen, vec, ids, off)
    got = gpu_search(idx, q, nprobe, k)
    res = check_against_oracle(cen, vec, ids, off, q, nprobe, k, got, storage)
    idx.close()
    return got, res


@pytest.mark.parametrize("nlist,dups", [
    (12, (3, 7)),                 # one coarse tile
    (100, (3, 40, 77)),           # three copies in three different tiles of 32 centroids
    (200, (31, 32, 63, 64, 199)), # copies on both sides of tile borders and in the last, partial tile
])
def test_duplicate_centroids_inside_at_and_past_the_boundary(nlist, dups):
    """The copies share one coarse score exactly (same operands, same order of operations).
    With `above` lists scoring higher, nprobe = above + m takes the m copies with the
    smallest list numbers, in ascending order, for every m."""
    d = 16
    above = 4
    alphas = np.linspace(0.1, 0.5, nlist)
    rng = np.random.default_rng(nlist)
    alphas = alphas[rng.permutation(nlist)]
    others = [j for j in range(nlist) if j not in dups]
    top = rng.choice(others, size=above, replace=False)
    alphas[top] = [2.0, 1.9, 1.8, 1.7]          # clearly ahead of the copies
    alphas[list(dups)] = 1.25                   # clearly ahead of the rest
    cen, vec, ids, off, u = _graded_index(nlist, d, alphas, seed=7 + nlist)
    q = np.stack([u, 2.5 * u, u]).astype(np.float32)
    q[2, 5] = 0.75                               # a component no centroid has: same coarse order
    for m in range(0, len(dups) + 2):
        nprobe = above + m
        say(f"duplicate centroids {dups} of {nlist}: nprobe={nprobe} ({min(m, len(dups))} of the copies inside)")
        got, res = _run(cen, vec, ids, off, q, nprobe, k=10)
        g_probes, g_coarse = got[2], got[3]
        for c in dups[1:]:
            assert np.array_equal(g_coarse[:, c], g_coarse[:, dups[0]])          # exact ties on the GPU
        want = O.probe_select(O.coarse(q, cen), nprobe)
        assert np.array_equal(g_probes, want)                                    # sets AND order
        assert res["probe_sets_equal"]
        inside = sorted(dups)[:min(m, len(dups))]
        for r in range(q.shape[0]):
            assert g_probes[r, :above].tolist() == top.tolist()
            assert g_probes[r, above:above + len(inside)].tolist() == inside     # smaller list numbers first


def test_ties_fp32_cannot_resolve_make_the_oracle_rescan_the_gpu_probe_set():
    """Centroids a < b with <q,a> = 1 and <q,b> = 1 + 2^-30: fp64 prefers b, any fp32
    accumulation rounds both to 1.0 and the tie goes to the smaller list a.  With the
    boundary between them the probe sets differ by a near-tie (far inside 1e-5 relative):
    accepted, and the oracle's scan runs over the GPU's set."""
    nlist, d = 40, 16
    alphas = np.linspace(0.1, 0.6, nlist)
    a, b = 9, 33                                  # different coarse tiles
    alphas[[2, 20]] = [3.0, 2.0]
    alphas[[a, b]] = 1.0
    cen, vec, ids, off, u = _graded_index(nlist, d, alphas, seed=11, extra_dim={b: 2.0 ** -30})
    q = u[None, :].copy()
    q[0, 1] = 1.0                                 # <q, b> = 1 + 2^-30, <q, a> = 1
    o_coarse = O.coarse(q, cen)
    assert o_coarse[0, b] > o_coarse[0, a] and o_coarse[0, b] - o_coarse[0, a] < 1e-8
    assert O.probe_select(o_coarse, 3)[0].tolist() == [2, 20, b]
    say("unresolvable tie at the boundary: nprobe=3")
    got, res = _run(cen, vec, ids, off, q, 3, k=12)
    assert got[3][0, a] == got[3][0, b] == np.float32(1.0)
    assert got[2][0].tolist() == [2, 20, a]       # GPU: tie -> smaller list
    assert res["probe_sets_equal"] is False       # the oracle re-scanned the GPU's probe set
    # the returned ids come from lists 2, 20 and a, none from b
    lists_of = np.searchsorted(off, np.arange(len(ids)), side="right") - 1
    pos = {int(i): p for p, i in enumerate(ids)}
    assert {int(lists_of[pos[int(i)]]) for i in got[0][0]} <= {2, 20, a}
    say("unresolvable tie inside the probe set: nprobe=4")
    got, res = _run(cen, vec, ids, off, q, 4, k=12)
    assert sorted(got[2][0].tolist()) == [2, a, 20, b] and res["probe_sets_equal"]
    # a swap beyond a near-tie is still rejected by the rules
    bad = got[2].copy()
    bad[0, -1] = 0
    with pytest.raises(AssertionError):
        CK.check_probes(bad, o_coarse, 4)


@pytest.mark.parametrize("rel", [1e-6, 3e-7, -1e-6])
def test_centroids_within_1e6_relative_of_the_boundary_score(rel):
    """The (nprobe+1)-th centroid scores within 1e-6 relative of the nprobe-th (on either
    side): fp32 may or may not order them like fp64; either probe set is accepted and the
    results must match the oracle's scan of the set that was used."""
    nlist, d = 70, 32
    rng = np.random.default_rng(5)
    alphas = rng.uniform(0.1, 0.6, nlist)
    alphas[[50, 8, 61]] = [1.5, 1.4, 1.3]
    alphas[12] = 1.1
    alphas[44] = 1.1 * (1.0 + rel)
    cen, vec, ids, off, u = _graded_index(nlist, d, alphas, seed=13, storage=np.float16)
    q = np.stack([u, 0.3 * u]).astype(np.float32)
    q[:, 3:] = rng.standard_normal((2, d - 3)).astype(np.float32) * 0.5       # orthogonal to every centroid
    say(f"near-tie at the boundary, relative gap {rel:g}: nprobe=4")
    got, res = _run(cen, vec, ids, off, q, 4, k=25, storage="fp16")
    for r in range(2):
        assert got[2][r, :3].tolist() == [50, 8, 61] and got[2][r, 3] in (12, 44)
    say(f"near-tie inside the probe set, relative gap {rel:g}: nprobe=5")
    got, res = _run(cen, vec, ids, off, q, 5, k=25, storage="fp16")
    assert res["probe_sets_equal"]
    for r in range(2):
        assert sorted(got[2][r].tolist()) == [8, 12, 44, 50, 61]
