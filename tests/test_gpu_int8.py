"""GPU parity for compressed lists (int8 codes with one fp32 scale per vector): the HIP
path through the C ABI against the CPU oracle on the same uploaded records, at small sizes
element by element (ragged and empty lists, shared lists, d from 16 to 768, every
placement) and at the sizes of the benchmark's C3 and C5 indexes."""
import numpy as np
import pytest

from oracle import check as CK
from oracle import ivf_oracle as O
from paper_2504_15302_amd import ivf
from paper_2504_15302_amd import workloads as W
from tests.gpu_util import DeviceWorkload, check_against_oracle, check_large, gpu_search, say, upload_host_index

pytestmark = pytest.mark.gpu


def _random_records(seed, n, d, nlist, empty_lists=(), spread=True):
    rng = np.random.default_rng(seed)
    cen = rng.standard_normal((nlist, d)).astype(np.float32)
    x = rng.standard_normal((n, d)).astype(np.float32)
    if spread:
        x *= rng.uniform(0.05, 20.0, size=(n, 1)).astype(np.float32)     # scales far apart
    sc = x.astype(np.float64) @ cen.astype(np.float64).T
    sc[:, list(empty_lists)] = -np.inf
    lab = np.argmax(sc, axis=1)
    order = np.argsort(lab, kind="stable")
    x, lab = x[order], lab[order]
    off = np.zeros(nlist + 1, dtype=np.int64)
    np.cumsum(np.bincount(lab, minlength=nlist), out=off[1:])
    ids = rng.permutation(5 * n + 3)[:n].astype(np.int64)
    return cen, W.quantize_int8_host(x), ids, off


def _floor(q, rec):
    codes, scales = W.split_int8_records(rec)
    nrm = np.linalg.norm(codes.astype(np.float32), axis=1) * scales
    return float(np.linalg.norm(q, axis=1).max() * nrm.max())


@pytest.fixture(scope="module")
def c1q():
    w = W.CONFIGS["C1-int8"]
    h = W.build_host_index(w)
    say("C1-int8: uploading 100k records of 384 codes + scale")
    return w, h, upload_host_index(h)


def test_c1_int8_matches_oracle(c1q):
    w, h, idx = c1q
    info = idx.info()
    assert info.dtype == ivf.IVF_INT8 and info.index_bytes == int(((np.diff(h.offsets) + 63) // 64).sum()) * 64 * (w.d + 4)
    q = W.queries(w)
    say("C1-int8: search nq=16 nprobe=8 k=10")
    got = gpu_search(idx, q, w.nprobe, w.k)
    res = check_against_oracle(h.centroids, h.vectors, h.ids, h.offsets, q, w.nprobe, w.k, got, "int8")
    say(f"C1-int8 ok: {res}")
    st = idx.last_search_stats()
    assert st.scan_bytes == st.scanned_vectors * (w.d + 4)
    for k, nprobe, nq in ((1, 1, 1), (5, 3, 7), (100, 8, 16), (1024, 256, 3), (129, 40, 70)):
        q = W.queries(w, batch=3, nq=nq)
        say(f"C1-int8: nq={nq} nprobe={nprobe} k={k}")
        got = gpu_search(idx, q, nprobe, k)
        check_against_oracle(h.centroids, h.vectors, h.ids, h.offsets, q, nprobe, k, got, "int8")
    for l in (0, 100, 255):
        rec, ids = idx.read_list(l, w.d, ivf.IVF_INT8)
        assert np.array_equal(rec, h.vectors[h.offsets[l]:h.offsets[l + 1]])
        assert np.array_equal(ids, h.ids[h.offsets[l]:h.offsets[l + 1]])


def test_c1_int8_results_do_not_depend_on_placement(c1q):
    w, h, idx = c1q
    q = W.queries(w, batch=6)
    ref = gpu_search(idx, q, w.nprobe, w.k)
    total = idx.info().index_bytes
    try:
        for direct in (1, 0):
            idx.set_option("host_direct", direct)
            for frac in (0.3, 0.0):
                say(f"C1-int8 budget {frac:.2f}, host lists {'read in place' if direct else 'staged'}")
                idx.set_device_budget(int(total * frac))
                got = gpu_search(idx, q, w.nprobe, w.k)
                assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])
                assert idx.last_search_stats().scan_bytes_streamed > 0
        say("C1-int8 budget back to everything, in the background")
        idx.set_option("host_direct", 1)
        idx.set_device_budget_async(2**62)
        while idx.budget_progress()[2]:
            got = gpu_search(idx, q, w.nprobe, w.k)
            assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])
    finally:
        idx.budget_wait()
        idx.set_option("host_direct", 1)
        idx.set_device_budget(2**62)
    rec, _ = idx.read_list(7, w.d, ivf.IVF_INT8)
    assert np.array_equal(rec, h.vectors[h.offsets[7]:h.offsets[7 + 1]])


CASES = [
    # name, n, d, nlist, empty lists, nq, nprobe, k
    ("d16_tiny_lists", 300, 16, 20, (3,), 9, 5, 7),
    ("d48_ragged", 5000, 48, 13, (), 33, 4, 10),
    ("d256_one_group_exactly", 3000, 256, 7, (0, 6), 5, 7, 64),
    ("d272_group_plus_one_chunk", 2500, 272, 6, (), 6, 3, 20),
    ("d768_three_groups", 4000, 768, 10, (4,), 12, 3, 100),
    ("d1024_k_above_candidates", 700, 1024, 9, (), 4, 2, 300),
    ("one_list_many_queries", 2000, 64, 1, (), 70, 1, 10),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_int8_edge_cases_match_oracle(case):
    name, n, d, nlist, empty, nq, nprobe, k = case
    cen, rec, ids, off = _random_records(sum(map(ord, name)), n, d, nlist, empty)
    rng = np.random.default_rng(1)
    q = rng.standard_normal((nq, d)).astype(np.float32)
    idx = ivf.Index()
    idx.upload(cen, rec, ids, off)
    say(f"int8 {name}: n={n} d={d} nlist={nlist} nq={nq} nprobe={nprobe} k={k}")
    got = gpu_search(idx, q, nprobe, k)
    check_against_oracle(cen, rec, ids, off, q, nprobe, k, got, "int8", abs_floor=_floor(q, rec))
    for option, value in (("scan_unroll", 8), ("scan_waves", 8), ("scan_waves", 1)):
        idx.set_option(option, value)
        again = gpu_search(idx, q, nprobe, k)
        assert np.array_equal(again[0], got[0]) and np.array_equal(again[1], got[1]), option
    idx.close()


def test_int8_extreme_codes_and_signs():
    """All codes at -127 or +127, and scales spanning 2^-20 .. 2^20: the sign extension of
    every byte position and the scale multiplication, against hand-computed values."""
    d, n = 32, 130
    rng = np.random.default_rng(3)
    codes = rng.choice(np.array([-127, 127], dtype=np.int8), size=(n, d))
    codes[0] = 127
    codes[1] = -127
    scales = (2.0 ** rng.integers(-20, 21, size=n)).astype(np.float32)
    scales[0] = scales[1] = 1.0
    rec = np.empty((n, d + 4), dtype=np.uint8)
    rec[:, :d] = codes.view(np.uint8)
    rec[:, d:] = scales.view(np.uint8).reshape(n, 4)
    cen = np.ones((1, d), dtype=np.float32)
    off = np.array([0, n], dtype=np.int64)
    ids = np.arange(n, dtype=np.int64)
    q = np.zeros((d + 1, d), dtype=np.float32)
    q[:d] = np.eye(d, dtype=np.float32)           # query t reads code t alone
    q[d] = 1.0
    idx = ivf.Index()
    idx.upload(cen, rec, ids, off)
    got = gpu_search(idx, q, 1, n)
    exact = (q.astype(np.float64) @ codes.astype(np.float64).T) * scales.astype(np.float64)[None, :]
    for r in range(d + 1):
        by_id = np.empty(n)
        by_id[got[0][r]] = got[1][r]
        assert np.array_equal(by_id, exact[r].astype(np.float32)), f"query {r}"     # sums of at most 32 small integers: exact in fp32
    check_against_oracle(cen, rec, ids, off, q, 1, n, got, "int8")
    idx.close()


def test_int8_rejects_d_not_a_multiple_of_16():
    cen = np.zeros((2, 24), dtype=np.float32)
    rec = np.zeros((4, 28), dtype=np.uint8)
    idx = ivf.Index()
    with pytest.raises(ivf.IvfError) as e:
        idx.upload(cen, rec, np.arange(4, dtype=np.int64), np.array([0, 2, 4], dtype=np.int64))
    assert e.value.code == -5
    idx.close()


def test_c3_int8_full_size_matches_oracle():
    w = W.CONFIGS["C3-int8"]
    dw = DeviceWorkload(w)
    q = W.queries(w)
    say("C3-int8: search nq=64 nprobe=64 k=20")
    got = gpu_search(dw.index, q, w.nprobe, w.k)
    res = check_large(dw, q, w.nprobe, w.k, got)
    say(f"C3-int8 ok: {res}")
    vec, ids, coff, cmap = dw.host_lists([5, 9000])
    for l in (5, 9000):
        rec, i = dw.index.read_list(l, w.d, ivf.IVF_INT8)
        c = cmap[l]
        assert np.array_equal(rec, vec[coff[c]:coff[c + 1]]) and np.array_equal(i, ids[coff[c]:coff[c + 1]])
    nblk = (np.diff(dw.off) + 63) // 64
    assert dw.index.info().index_bytes == int(nblk.sum()) * 64 * (w.d + 4)   # about half of the fp16 index
    dw.index.close()


def test_c5_int8_full_size_every_row_matches_oracle():
    w = W.CONFIGS["C5-int8"]
    dw = DeviceWorkload(w, groups_per_chunk=32)
    q = W.queries(w)
    say("C5-int8: search nq=128 nprobe=128 k=100")
    got = gpu_search(dw.index, q, w.nprobe, w.k)
    res = check_large(dw, q, w.nprobe, w.k, got)
    assert res["queries"] == w.nq
    say(f"C5-int8 ok on all {w.nq} rows: {res}")
    dw.index.close()
