"""Pins for the CPU oracle: each test fixes it to something other than itself — a
library routine on a special case, a hand-written closed form, or an invariant of
the definition (similarity match + top-k, paper Sections 2.2 and 6.1; IVF-Flat /
inner product per the benchmark configurations)."""
import numpy as np
import pytest

from oracle import ivf_oracle as O
from oracle import check as CK
from paper_2504_15302_amd import workloads as W
from tests.golden_util import load_basis_case


def _tiny(seed, n=600, d=24, nlist=12, nq=7, storage=np.float32, normalise=True):
    rng = np.random.default_rng(seed)
    cen = rng.standard_normal((nlist, d)).astype(np.float32)
    x = rng.standard_normal((n, d)).astype(np.float32)
    q = rng.standard_normal((nq, d)).astype(np.float32)
    if normalise:
        cen /= np.linalg.norm(cen, axis=1, keepdims=True)
        x /= np.linalg.norm(x, axis=1, keepdims=True)
        q /= np.linalg.norm(q, axis=1, keepdims=True)
    lab = np.argmax(x.astype(np.float64) @ cen.astype(np.float64).T, axis=1)
    order = np.argsort(lab, kind="stable")
    x, lab = x[order], lab[order]
    off = np.zeros(nlist + 1, dtype=np.int64)
    np.cumsum(np.bincount(lab, minlength=nlist), out=off[1:])
    ids = rng.permutation(10 * n)[:n].astype(np.int64)
    return cen, np.ascontiguousarray(x.astype(storage)), ids, off, q


def _brute(x, ids, q, k):
    """Library fp64 matmul + full sort by (score desc, id asc) over ALL vectors."""
    s = q.astype(np.float64) @ x.astype(np.float64).T
    out_i = np.full((q.shape[0], k), -1, dtype=np.int64)
    out_s = np.full((q.shape[0], k), -np.inf)
    for r in range(q.shape[0]):
        o = np.lexsort((ids, -s[r]))[:k]
        out_i[r, :len(o)] = ids[o]
        out_s[r, :len(o)] = s[r, o]
    return out_i, out_s


def test_half_decoder_matches_numpy_on_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([O.half_to_double(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("storage", [np.float32, np.float16])
@pytest.mark.parametrize("k", [1, 5, 10, 700])
def test_all_lists_probed_equals_exhaustive_search(seed, storage, k):
    cen, x, ids, off, q = _tiny(seed, storage=storage)
    oi, os_, pr, _ = O.search(cen, x, ids, off, q, nprobe=cen.shape[0], kout=k)
    bi, bs = _brute(x, ids, q, k)
    assert np.array_equal(oi, bi)
    fin = np.isfinite(bs)
    assert np.array_equal(np.isfinite(os_), fin)
    assert np.allclose(os_[fin], bs[fin], rtol=1e-12, atol=1e-14)
    assert sorted(pr[0].tolist()) == list(range(cen.shape[0]))


@pytest.mark.parametrize("seed", range(3))
def test_inner_product_ranking_equals_library_l2_knn_on_unit_vectors(seed):
    """For unit vectors |q-x|^2 = 2 - 2<q,x>: the IP ranking is the ascending-L2
    ranking, which a library brute-force k-NN computes independently."""
    from sklearn.neighbors import NearestNeighbors
    cen, x, ids, off, q = _tiny(100 + seed, n=500, d=16)
    k = 8
    oi, _, _, _ = O.search(cen, x, ids, off, q, nprobe=cen.shape[0], kout=k)
    nn = NearestNeighbors(n_neighbors=k, algorithm="brute", metric="euclidean").fit(x.astype(np.float64))
    _, idx = nn.kneighbors(q.astype(np.float64))
    assert np.array_equal(oi, ids[idx])


@pytest.mark.parametrize("storage", [np.float32, np.float16])
def test_closed_form_basis_case_from_golden_file(storage):
    g = load_basis_case(storage)
    for e in g["expects"]:
        q = g["queries"][e["query"]][None, :]
        oi, os_, pr, cs = O.search(g["centroids"], g["vectors"], g["ids"], g["offsets"], q,
                                   nprobe=e["nprobe"], kout=e["k"])
        assert pr[0].tolist() == e["probes"], e
        assert oi[0].tolist() == e["ids"], e
        assert os_[0].tolist() == e["scores"], e
        assert cs[0].tolist() == q[0].astype(np.float64).tolist()


def test_every_returned_score_is_the_dot_product_of_its_vector():
    cen, x, ids, off, q = _tiny(7, n=900, d=40)
    oi, os_, pr, _ = O.search(cen, x, ids, off, q, nprobe=4, kout=9)
    pos = {int(u): i for i, u in enumerate(ids)}
    for r in range(q.shape[0]):
        for c in range(9):
            want = np.dot(q[r].astype(np.float64), x[pos[int(oi[r, c])]].astype(np.float64))
            assert abs(os_[r, c] - want) <= 1e-13 * max(1.0, abs(want))


def test_invariants_on_c1_shaped_workload():
    w = W.scaled(W.CONFIGS["C1"], n=20_000, nlist=64)
    h = W.build_host_index(w)
    q = W.queries(w)
    oi, os_, pr, cs = O.search(h.centroids, h.vectors, h.ids, h.offsets, q, w.nprobe, w.k + 1)
    assert np.all(os_[:, :-1] >= os_[:, 1:])
    for r in range(q.shape[0]):
        assert len(set(oi[r].tolist())) == oi.shape[1]
    CK.check_ids_in_probed_lists(oi, pr, h.ids, h.offsets)
    # probes really are the nprobe best lists, best first, by an independent fp64 matmul
    ref = q.astype(np.float64) @ h.centroids.astype(np.float64).T
    assert np.allclose(cs, ref, rtol=1e-12, atol=1e-15)
    for r in range(q.shape[0]):
        assert pr[r].tolist() == np.lexsort((np.arange(w.nlist), -ref[r]))[:w.nprobe].tolist()


def test_prefix_property_and_merge_property_of_selection():
    cen, x, ids, off, q = _tiny(11, n=1500, d=20, nlist=16)
    cs = O.coarse(q, cen)
    pr = O.probe_select(cs, 8)
    k = 12
    full_i, full_s = O.scan_select(x, ids, off, q, pr, k)
    for kk in (1, 3, 7):
        pi, ps = O.scan_select(x, ids, off, q, pr, kk)
        assert np.array_equal(pi, full_i[:, :kk]) and np.array_equal(ps, full_s[:, :kk])
    ai, as_ = O.scan_select(x, ids, off, q, pr[:, :3], k)
    bi, bs = O.scan_select(x, ids, off, q, pr[:, 3:], k)
    for r in range(q.shape[0]):
        ci = np.concatenate([ai[r], bi[r]])
        c_s = np.concatenate([as_[r], bs[r]])
        keep = ci >= 0
        o = np.lexsort((ci[keep], -c_s[keep]))[:k]
        assert np.array_equal(ci[keep][o], full_i[r]) and np.array_equal(c_s[keep][o], full_s[r])


def test_monotone_in_nprobe_and_full_recall_at_nlist():
    cen, x, ids, off, q = _tiny(13, n=2000, d=16, nlist=20)
    k = 10
    bi, _ = _brute(x, ids, q, k)
    prev_s, prev_recall = None, -1.0
    for nprobe in (1, 2, 5, 10, 20):
        oi, os_, _, _ = O.search(cen, x, ids, off, q, nprobe, k)
        if prev_s is not None:
            assert np.all(os_ >= prev_s)
        prev_s = os_
        recall = np.mean([len(set(oi[r]) & set(bi[r])) / k for r in range(q.shape[0])])
        assert recall >= prev_recall
        prev_recall = recall
    assert prev_recall == 1.0


def test_probe_ties_go_to_the_smaller_list_and_nprobe_is_clamped():
    rng = np.random.default_rng(3)
    cen = rng.standard_normal((6, 8)).astype(np.float32)
    cen[4] = cen[1]                      # exact duplicate centroid
    q = (cen[1] * 2).reshape(1, -1).astype(np.float32)
    cs = O.coarse(q, cen)
    assert cs[0, 1] == cs[0, 4]
    pr = O.probe_select(cs, 6)[0].tolist()
    assert pr.index(1) + 1 == pr.index(4)
    x = rng.standard_normal((30, 8)).astype(np.float32)
    off = np.arange(0, 31, 5, dtype=np.int64)
    ids = np.arange(30, dtype=np.int64)
    _, _, pr2, _ = O.search(cen, x, ids, off, q, nprobe=99, kout=3)
    assert pr2.shape == (1, 6)


def test_score_ties_go_to_the_smaller_id_then_position():
    d = 8
    rng = np.random.default_rng(5)
    v = rng.standard_normal(d).astype(np.float32)
    x = np.stack([v, v, v * 0.5, v]).astype(np.float32)
    ids = np.array([9, 4, 1, 4], dtype=np.int64)     # duplicate id 4 on purpose
    off = np.array([0, 2, 4], dtype=np.int64)
    cen = np.stack([v, v]).astype(np.float32)
    oi, os_, _, _ = O.search(cen, x, ids, off, v[None, :], nprobe=2, kout=5)
    assert oi[0].tolist() == [4, 4, 9, 1, -1]
    assert os_[0, 0] == os_[0, 1] == os_[0, 2] and np.isneginf(os_[0, 4])


def test_assign_matches_library_argmax_and_breaks_ties_low():
    rng = np.random.default_rng(17)
    cen = rng.standard_normal((9, 12)).astype(np.float32)
    cen[7] = cen[2]
    x = rng.standard_normal((300, 12)).astype(np.float32)
    x[0] = cen[2]
    lab, best = O.assign(x, cen)
    s = x.astype(np.float64) @ cen.astype(np.float64).T
    assert np.array_equal(lab, np.argmax(s, axis=1))
    assert lab[0] == 2
    assert np.allclose(best, s.max(axis=1), rtol=1e-12)
    lab16, _ = O.assign(x.astype(np.float16), cen)
    s16 = x.astype(np.float16).astype(np.float64) @ cen.astype(np.float64).T
    assert np.array_equal(lab16, np.argmax(s16, axis=1))


def test_rows_do_not_depend_on_batch_or_on_order_inside_a_list_or_on_list_labels():
    cen, x, ids, off, q = _tiny(19, n=1200, d=16, nlist=10)
    k, nprobe = 6, 3
    oi, os_, _, _ = O.search(cen, x, ids, off, q, nprobe, k)
    for r in (0, 3):
        si, ss, _, _ = O.search(cen, x, ids, off, q[r:r + 1], nprobe, k)
        assert np.array_equal(si[0], oi[r]) and np.array_equal(ss[0], os_[r])
    # reverse the order of the vectors inside every list
    perm = np.concatenate([np.arange(off[j], off[j + 1])[::-1] for j in range(len(off) - 1)])
    pi, ps, _, _ = O.search(cen, x[perm], ids[perm], off, q, nprobe, k)
    assert np.array_equal(pi, oi) and np.array_equal(ps, os_)
    # relabel the lists (reverse their order)
    nl = len(off) - 1
    lperm = np.arange(nl)[::-1]
    rows = np.concatenate([np.arange(off[j], off[j + 1]) for j in lperm])
    off2 = np.zeros_like(off)
    np.cumsum(np.diff(off)[lperm], out=off2[1:])
    ri, rs, _, _ = O.search(cen[lperm], x[rows], ids[rows], off2, q, nprobe, k)
    assert np.array_equal(ri, oi) and np.array_equal(rs, os_)


def test_generator_closed_forms_and_assignment_equals_component():
    """Mixture closed forms: E<mu_c,x> ~ 1/sqrt(1+sigma^2 d); same-component pairs
    ~ 1/(1+sigma^2 d); and the component a vector was drawn from is its arg-max
    inner-product centroid (all of C1)."""
    w = W.CONFIGS["C1"]
    h = W.build_host_index(w)
    lab = W.list_labels(h.offsets)
    got, best = O.assign(h.vectors, h.centroids)
    assert np.array_equal(got, lab)
    want = 1.0 / np.sqrt(1.0 + w.sigma ** 2 * w.d)
    assert abs(best.mean() - want) < 2e-3
    a = h.vectors[h.offsets[5]:h.offsets[5] + 200].astype(np.float64)
    pair = (a @ a.T)[np.triu_indices(200, 1)].mean()
    assert abs(pair - want ** 2) < 5e-3
    assert abs(np.linalg.norm(h.vectors[:1000].astype(np.float64), axis=1) - 1).max() < 1e-6
    assert sorted(h.ids.tolist()) == list(range(w.n))
    assert abs(np.diff(h.offsets).mean() - w.n / w.nlist) < 1e-9
    q8 = W.queries(w, nq=8)
    assert np.array_equal(q8, W.queries(w)[:8])
    assert not np.array_equal(W.queries(w, batch=1), W.queries(w))


def test_fp16_storage_stays_within_the_fp16_score_bar_of_fp32_storage():
    w = W.scaled(W.CONFIGS["C1"], n=20_000, nlist=64)
    h = W.build_host_index(w)
    q = W.queries(w)
    i32, s32, _, _ = O.search(h.centroids, h.vectors, h.ids, h.offsets, q, w.nprobe, w.k)
    i16, s16, _, _ = O.search(h.centroids, h.vectors.astype(np.float16), h.ids, h.offsets, q, w.nprobe, w.k)
    assert np.abs(s16 - s32).max() / np.abs(s32).max() < 1e-3


def test_checker_accepts_near_tie_swaps_and_rejects_real_differences():
    ref_i = np.array([[5, 6, 7, 8]], dtype=np.int64)
    ref_s = np.array([[1.0, 0.5, 0.5 - 1e-7, 0.2]])
    ok_i = np.array([[5, 7, 6]], dtype=np.int64)
    ok_s = np.array([[1.0, 0.5, 0.5]], dtype=np.float32)
    assert CK.check_topk(ok_i, ok_s, ref_i, ref_s, 3, 1e-5)["tie_runs_reordered"] == 1
    with pytest.raises(AssertionError):
        CK.check_topk(np.array([[5, 8, 6]]), ok_s, ref_i, ref_s, 3, 1e-5)
    with pytest.raises(AssertionError):
        CK.check_topk(np.array([[5, 6, 7]]), np.array([[1.0, 0.5, 0.4]], dtype=np.float32),
                      ref_i, ref_s, 3, 1e-5)
    # boundary: the (k+1)-th may stand in for the k-th only when they nearly tie
    CK.check_topk(np.array([[5, 7]]), np.array([[1.0, 0.5]], dtype=np.float32), ref_i, ref_s, 2, 1e-5)
    with pytest.raises(AssertionError):
        CK.check_topk(np.array([[5, 6, 8]]), np.array([[1.0, 0.5, 0.2]], dtype=np.float32),
                      ref_i, ref_s, 3, 1e-5)
    cs = np.array([[0.9, 0.5, 0.5 + 1e-8, 0.1]])
    assert CK.check_probes(np.array([[0, 2]]), cs, 2) is True
    assert CK.check_probes(np.array([[0, 1]]), cs, 2) is False
    with pytest.raises(AssertionError):
        CK.check_probes(np.array([[0, 3]]), cs, 2)
