"""Pins for the oracle's int8 storage (compressed lists: d signed codes and one fp32 scale
per vector, the stored vector being scale * codes) and for the quantiser that prepares
such records.  The paper only points at compressed / on-disk indexes as the way to trade
memory for accuracy (Section 6.5 "On-Disk Index"); the format is this build's reading, so
the pins are mathematical: exhaustive search with a library matmul, re-derived scores,
reduction to the float32 routine where the codes are the vector, and the quantiser's
error bound."""
import numpy as np
import pytest

from oracle import ivf_oracle as O
from paper_2504_15302_amd import workloads as W
from tests.golden_util import load_basis_case
from tests.test_oracle_pins import _brute, _tiny


def _records(codes: np.ndarray, scales: np.ndarray) -> np.ndarray:
    rows, d = codes.shape
    rec = np.empty((rows, d + 4), dtype=np.uint8)
    rec[:, :d] = codes.astype(np.int8).view(np.uint8)
    rec[:, d:] = scales.astype(np.float32).view(np.uint8).reshape(rows, 4)
    return rec


@pytest.mark.parametrize("seed,k", [(0, 1), (1, 5), (2, 10), (3, 40)])
def test_all_lists_probed_equals_exhaustive_search_over_dequantised_vectors(seed, k):
    cen, x, ids, off, q = _tiny(seed, n=700, d=32, nlist=9)
    rec = W.quantize_int8_host(x)
    codes, scales = W.split_int8_records(rec)
    assert (codes < 0).any() and (codes > 0).any()            # signs matter in what follows
    xhat = codes.astype(np.float64) * scales.astype(np.float64)[:, None]
    bi, bs = _brute(xhat, ids, q, k)
    oi, os_, _, _ = O.search(cen, rec, ids, off, q, nprobe=9, kout=k)
    assert np.array_equal(oi, bi)
    assert np.allclose(os_, bs, rtol=1e-13, atol=1e-15)


def test_every_returned_score_is_scale_times_the_dot_product_with_the_codes():
    cen, x, ids, off, q = _tiny(11, n=900, d=48)
    rec = W.quantize_int8_host(3.0 * x)                        # scales away from the unit range
    codes, scales = W.split_int8_records(rec)
    oi, os_, pr, _ = O.search(cen, rec, ids, off, q, nprobe=4, kout=9)
    pos = {int(u): i for i, u in enumerate(ids)}
    for r in range(q.shape[0]):
        for c in range(9):
            i = pos[int(oi[r, c])]
            want = float(scales[i]) * np.dot(q[r].astype(np.float64), codes[i].astype(np.float64))
            assert abs(os_[r, c] - want) <= 1e-13 * max(1.0, abs(want))


def test_integer_vectors_with_unit_scale_reduce_to_the_float32_routine():
    rng = np.random.default_rng(5)
    nlist, d, n = 6, 16, 300
    cen = rng.standard_normal((nlist, d)).astype(np.float32)
    codes = rng.integers(-127, 128, size=(n, d)).astype(np.int8)
    off = np.linspace(0, n, nlist + 1).astype(np.int64)
    ids = rng.permutation(n).astype(np.int64)
    q = rng.standard_normal((5, d)).astype(np.float32)
    a = O.search(cen, _records(codes, np.ones(n)), ids, off, q, nprobe=3, kout=12)
    b = O.search(cen, codes.astype(np.float32), ids, off, q, nprobe=3, kout=12)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    # and a power-of-two scale only shifts the exponent
    c = O.search(cen, _records(codes, np.full(n, 0.25)), ids, off, q, nprobe=3, kout=12)
    assert np.array_equal(c[0], b[0]) and np.array_equal(c[1], 0.25 * b[1])


def test_closed_form_basis_case_survives_quantisation():
    """One non-zero coordinate per vector: code 127 and scale a/127, so the stored vector
    is the original up to one float32 rounding of the scale."""
    g = load_basis_case(np.float32)
    rec = W.quantize_int8_host(g["vectors"])
    codes, scales = W.split_int8_records(rec)
    assert set(np.unique(np.abs(codes))) <= {0, 127}
    for e in g["expects"]:
        q = g["queries"][e["query"]][None, :]
        oi, os_, pr, _ = O.search(g["centroids"], rec, g["ids"], g["offsets"], q, nprobe=e["nprobe"], kout=e["k"])
        assert pr[0].tolist() == e["probes"] and oi[0].tolist() == e["ids"], e
        fin = np.isfinite(e["scores"])
        assert np.allclose(os_[0][fin], np.array(e["scores"])[fin], rtol=2e-7, atol=0)
        assert np.array_equal(np.isfinite(os_[0]), fin)


def test_quantiser_properties_and_score_error_bound():
    rng = np.random.default_rng(9)
    x = rng.standard_normal((500, 96)).astype(np.float32) * rng.uniform(0.01, 30, size=(500, 1)).astype(np.float32)
    x[17] = 0.0
    rec = W.quantize_int8_host(x)
    assert rec.dtype == np.uint8 and rec.shape == (500, 100)
    codes, scales = W.split_int8_records(rec)
    assert codes.min() >= -127 and codes.max() <= 127
    nz = np.abs(x).max(axis=1) > 0
    assert (np.abs(codes[nz]).max(axis=1) == 127).all()       # the full range is used
    assert (codes[17] == 0).all() and scales[17] == 1.0
    assert np.allclose(scales[nz], np.abs(x[nz]).max(axis=1) / 127.0, rtol=1e-6)
    err = np.abs(x.astype(np.float64) - codes.astype(np.float64) * scales.astype(np.float64)[:, None])
    assert (err <= 0.5 * scales[:, None] * (1 + 1e-5)).all()   # round to nearest code
    q = rng.standard_normal((8, 96)).astype(np.float32)
    exact = q.astype(np.float64) @ x.astype(np.float64).T
    quant = (q.astype(np.float64) @ codes.astype(np.float64).T) * scales.astype(np.float64)[None, :]
    bound = 0.5 * np.abs(q).sum(axis=1)[:, None] * scales[None, :]
    assert (np.abs(quant - exact) <= bound * (1 + 1e-5) + 1e-12).all()


def test_int8_workload_keeps_the_top_results_of_the_float_workload():
    """On the benchmark's mixture (C1 shape, scaled down) the quantisation error per score,
    at most (scale/2)*|q|_1, is far below the gap between a query's own cluster and the
    others: the best result and the bulk of the top-10 stay put."""
    w = W.scaled(W.CONFIGS["C1"], n=20000, name="C1-small")
    wq = W.scaled(W.CONFIGS["C1-int8"], n=20000, name="C1-int8-small")
    h, hq = W.build_host_index(w), W.build_host_index(wq)
    assert hq.vectors.dtype == np.uint8 and hq.vectors.shape == (w.n, w.d + 4)
    assert np.array_equal(h.offsets, hq.offsets) and np.array_equal(h.ids, hq.ids)
    q = W.queries(w)
    a = O.search(h.centroids, h.vectors, h.ids, h.offsets, q, w.nprobe, w.k)
    b = O.search(hq.centroids, hq.vectors, hq.ids, hq.offsets, q, w.nprobe, w.k)
    assert np.array_equal(a[2], b[2])                          # probes do not depend on the storage
    assert np.abs(a[1] - b[1]).max() < 5e-3
    overlap = np.mean([len(set(a[0][r]) & set(b[0][r])) / w.k for r in range(q.shape[0])])
    assert overlap >= 0.8
