"""Pins for the product-quantisation oracle (oracle/pq_oracle.py) and for the encoder of
the workload generator: each fixes them to something other than themselves."""
import os

import numpy as np
import pytest

from oracle import ivf_oracle as O
from oracle import pq_oracle as PQ
from paper_2504_15302_amd import workloads as W

HERE = os.path.dirname(os.path.abspath(__file__))


def _tiny(seed, n=500, d=24, M=6, nlist=9, nq=5):
    rng = np.random.default_rng(seed)
    cen = rng.standard_normal((nlist, d)).astype(np.float32)
    x = rng.standard_normal((n, d)).astype(np.float32)
    q = rng.standard_normal((nq, d)).astype(np.float32)
    cb = rng.standard_normal((M, 256, d // M)).astype(np.float32)
    lab = np.argmax(x.astype(np.float64) @ cen.astype(np.float64).T, axis=1)
    o = np.argsort(lab, kind="stable")
    x, lab = x[o], lab[o]
    off = np.zeros(nlist + 1, dtype=np.int64)
    np.cumsum(np.bincount(lab, minlength=nlist), out=off[1:])
    ids = rng.permutation(9 * n)[:n].astype(np.int64)
    codes = W.pq_encode_host(x, cb)
    return cen, x, codes, cb, ids, off, q


def test_hand_worked_case():
    vals = {}
    for line in open(os.path.join(HERE, "golden", "pq_case.txt")):
        t = line.split()
        if t and not t[0].startswith("#"):
            vals[t[0]] = [float(v) for v in t[1:]]
    cb = np.zeros((2, 256, 2), dtype=np.float32)
    cb[0, :3] = [[1, 0], [0, 2], [-1, -1]]
    cb[1, :3] = [[0.5, 0], [0, -3], [2, 2]]
    codes = np.array(vals["codes"], dtype=np.uint8).reshape(-1, 2)
    ids = np.array(vals["ids"], dtype=np.int64)
    q = np.array([vals["query"]], dtype=np.float32)
    T = PQ.adc_tables(q[0], cb)
    assert T[0, :3].tolist() == vals["table0"] and T[1, :3].tolist() == vals["table1"]
    assert PQ.adc_scores(T, codes).tolist() == vals["scores"]
    cen = np.array([[1, 0, 0, 0]], dtype=np.float32)
    oi, os_, pr, _ = PQ.search(cen, codes, cb, ids, np.array([0, 5], dtype=np.int64), q, 1, 4)
    assert oi[0].tolist() == [int(v) for v in vals["top4_ids"]] and os_[0].tolist() == vals["top4_scores"]
    oi, os_, _, _ = PQ.search(cen, codes, cb, ids, np.array([0, 5], dtype=np.int64), q, 1, 7)
    assert oi[0].tolist() == [10, 13, 11, 14, 12, -1, -1] and np.isneginf(os_[0, 5:]).all()


@pytest.mark.parametrize("seed", range(5))
def test_table_scores_equal_a_library_matmul_against_the_decoded_vectors(seed):
    cen, x, codes, cb, ids, off, q = _tiny(seed)
    xhat = PQ.decode(codes, cb)
    want = q.astype(np.float64) @ xhat.astype(np.float64).T
    for r in range(q.shape[0]):
        got = PQ.adc_scores(PQ.adc_tables(q[r], cb), codes)
        assert np.allclose(got, want[r], rtol=0, atol=1e-12 * np.abs(want[r]).max())
    # decoding copies codebook entries: every slice of a decoded vector is a codeword
    for m in range(cb.shape[0]):
        dsub = cb.shape[2]
        assert np.array_equal(xhat[:, m * dsub:(m + 1) * dsub], cb[m][codes[:, m]])


@pytest.mark.parametrize("seed", range(4))
@pytest.mark.parametrize("k", [1, 10, 600])
def test_all_lists_probed_equals_exhaustive_search_over_the_decoded_vectors(seed, k):
    cen, x, codes, cb, ids, off, q = _tiny(10 + seed)
    oi, os_, pr, _ = PQ.search(cen, codes, cb, ids, off, q, nprobe=cen.shape[0], kout=k)
    xhat = PQ.decode(codes, cb).astype(np.float64)
    s = q.astype(np.float64) @ xhat.T
    for r in range(q.shape[0]):
        o = np.lexsort((ids, -s[r]))[:k]
        assert oi[r, :len(o)].tolist() == ids[o].tolist()
        assert np.allclose(os_[r, :len(o)], s[r, o], rtol=1e-12, atol=1e-12)
        assert (oi[r, len(o):] == -1).all()


@pytest.mark.parametrize("seed", range(3))
def test_matches_the_flat_oracle_on_the_decoded_vectors_for_any_nprobe(seed):
    """The decoded vectors are exact float32 values, so the flat fp32 oracle over them is
    the same search by another route (one long fp64 sum instead of M table entries)."""
    cen, x, codes, cb, ids, off, q = _tiny(20 + seed)
    xhat = PQ.decode(codes, cb)
    for nprobe in (1, 3, 9):
        oi, os_, pr, _ = PQ.search(cen, codes, cb, ids, off, q, nprobe, 12)
        fi, fs, fpr, _ = O.search(cen, xhat, ids, off, q, nprobe, 12)
        assert np.array_equal(pr, fpr) and np.array_equal(oi, fi)
        assert np.allclose(os_, fs, rtol=1e-12, atol=1e-12)


def test_codes_that_reproduce_their_vectors_reduce_to_the_flat_search_on_the_originals():
    """Codebooks that contain every stored slice: encoding loses nothing, and the PQ search
    is the flat search over the original vectors."""
    rng = np.random.default_rng(3)
    n, d, M = 200, 12, 3
    cb = rng.standard_normal((M, 256, d // M)).astype(np.float32)
    picks = rng.integers(0, 256, size=(n, M))
    x = np.concatenate([cb[m][picks[:, m]] for m in range(M)], axis=1).astype(np.float32)
    codes = W.pq_encode_host(x, cb)
    assert np.array_equal(PQ.decode(codes, cb), x)
    cen = rng.standard_normal((4, d)).astype(np.float32)
    off = np.array([0, 50, 50, 120, 200], dtype=np.int64)
    ids = rng.permutation(n).astype(np.int64)
    q = rng.standard_normal((6, d)).astype(np.float32)
    oi, os_, _, _ = PQ.search(cen, codes, cb, ids, off, q, 2, 9)
    fi, fs, _, _ = O.search(cen, x, ids, off, q, 2, 9)
    assert np.array_equal(oi, fi) and np.allclose(os_, fs, rtol=1e-12, atol=1e-12)


def test_encoder_is_the_nearest_codeword_and_obeys_its_error_bound():
    cen, x, codes, cb, ids, off, q = _tiny(7, n=300)
    M, _, dsub = cb.shape
    xhat = PQ.decode(codes, cb)
    for m in range(M):
        xm = x[:, m * dsub:(m + 1) * dsub].astype(np.float64)
        dist = ((xm[:, None, :] - cb[m][None, :, :].astype(np.float64)) ** 2).sum(axis=2)   # brute force
        best = dist.min(axis=1)
        mine = dist[np.arange(len(xm)), codes[:, m]]
        assert np.all(mine <= best * (1 + 1e-5) + 1e-6)
    # |<q, x^> - <q, x>| <= sum_m |q_m| |x_m - x^_m|
    err = np.abs(q.astype(np.float64) @ (xhat.astype(np.float64) - x.astype(np.float64)).T)
    bound = np.zeros_like(err)
    for m in range(M):
        sl = slice(m * dsub, (m + 1) * dsub)
        bound += np.linalg.norm(q[:, sl].astype(np.float64), axis=1)[:, None] * \
            np.linalg.norm((x[:, sl] - xhat[:, sl]).astype(np.float64), axis=1)[None, :]
    assert np.all(err <= bound + 1e-9)


def test_workload_generator_pq_variant():
    w = W.scaled(W.CONFIGS["C1-pq"], n=6000, nlist=24)
    h = W.build_host_index(w)
    cb = W.pq_codebooks(w)
    assert h.vectors.dtype == np.uint8 and h.vectors.shape == (w.n, w.pq_m) and cb.shape == (w.pq_m, 256, 8)
    assert w.row_bytes == w.pq_m == 48
    # the codes stand for vectors near the originals: same mixture, unit norm within 25 %
    xhat = PQ.decode(h.vectors[:500], cb)
    nrm = np.linalg.norm(xhat, axis=1)
    assert 0.75 < nrm.mean() < 1.25
    # and searching them still finds part of what the float32 index finds (the codebooks are
    # untrained samples, 8 dimensions per byte: a coarse approximation)
    w32 = W.scaled(W.CONFIGS["C1"], n=6000, nlist=24)
    h32 = W.build_host_index(w32)
    q = W.queries(w)
    assert np.array_equal(q, W.queries(w32))
    oi, _, _, _ = PQ.search(h.centroids, h.vectors, cb, h.ids, h.offsets, q, 4, 10)
    fi, _, _, _ = O.search(h32.centroids, h32.vectors, h32.ids, h32.offsets, q, 4, 10)
    overlap = np.mean([len(set(a) & set(b)) / 10 for a, b in zip(oi, fi)])
    assert overlap >= 0.15, overlap
