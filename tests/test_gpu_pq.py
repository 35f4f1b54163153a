"""GPU parity for lists stored as product-quantisation codes (IVF_PQ8): the HIP path through
the C ABI against the CPU oracles.  The codes stand for decoded float32 vectors, so the
search is exact over them; it is compared element by element with the PQ oracle (table
entries summed in fp64) and, through the shared helper, with the flat fp64 oracle over the
decoded vectors, under the benchmark's bar for exact storage (1e-5 relative)."""
import numpy as np
import pytest

from oracle import check as CK
from oracle import pq_oracle as PQ
from paper_2504_15302_amd import ivf
from paper_2504_15302_amd import workloads as W
from tests.gpu_util import DeviceWorkload, check_against_oracle, check_large, gpu_search, say

pytestmark = pytest.mark.gpu


def _upload(cen, codes, cb, ids, off):
    idx = ivf.Index()
    idx.set_pq_codebooks(cb)
    idx.upload(cen, codes, ids, off, dtype=ivf.IVF_PQ8)
    return idx


def _check(cen, codes, cb, ids, off, q, nprobe, k, got, abs_floor=0.0):
    xhat = PQ.decode(codes, cb)
    res = check_against_oracle(cen, xhat, ids, off, q, nprobe, k, got, "fp32", abs_floor=abs_floor)
    # and against the table-by-table oracle, on the probe sets the GPU used
    oi, os_ = PQ.scan_select(codes, cb, ids, off, q, got[2], k + 8)
    CK.check_topk(got[0], got[1], oi, os_, k, CK.SCORE_REL["pq8"], abs_floor=abs_floor)
    return res


@pytest.fixture(scope="module")
def c1pq():
    w = W.CONFIGS["C1-pq"]
    h = W.build_host_index(w)
    cb = W.pq_codebooks(w)
    say(f"C1-pq: uploading 100k vectors as {w.pq_m} code bytes each")
    idx = _upload(h.centroids, h.vectors, cb, h.ids, h.offsets)
    yield w, h, cb, idx
    idx.close()


def test_c1_pq_matches_oracle(c1pq):
    w, h, cb, idx = c1pq
    q = W.queries(w)
    say("C1-pq: search nq=16 nprobe=8 k=10")
    got = gpu_search(idx, q, w.nprobe, w.k)
    res = _check(h.centroids, h.vectors, cb, h.ids, h.offsets, q, w.nprobe, w.k, got)
    say(f"C1-pq ok: {res}")
    info = idx.info()
    assert info.dtype == ivf.IVF_PQ8 and info.index_bytes == int(((np.diff(h.offsets) + 63) // 64).sum()) * 64 * w.pq_m
    st = idx.last_search_stats()
    assert st.scan_bytes == st.scanned_vectors * w.pq_m
    for l in (0, 100, 255):
        codes, ids = idx.read_list(l, w.pq_m, ivf.IVF_PQ8)
        assert np.array_equal(codes, h.vectors[h.offsets[l]:h.offsets[l + 1]])
        assert np.array_equal(ids, h.ids[h.offsets[l]:h.offsets[l + 1]])


@pytest.mark.parametrize("k,nprobe,nq", [(1, 1, 1), (100, 8, 16), (1024, 256, 3), (20, 16, 200)])
def test_c1_pq_other_shapes_and_pruning(c1pq, k, nprobe, nq):
    w, h, cb, idx = c1pq
    q = W.queries(w, batch=2, nq=nq)
    try:
        for prune in (0, 2):
            idx.set_option("scan_prune", prune)
            say(f"C1-pq: nq={nq} nprobe={nprobe} k={k} scan_prune={prune}")
            got = gpu_search(idx, q, nprobe, k)
            if prune == 0:
                ref = got
                _check(h.centroids, h.vectors, cb, h.ids, h.offsets, q, nprobe, k, got)
            else:
                assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])
    finally:
        idx.set_option("scan_prune", 1)


def test_c1_pq_placement_queued_and_noalloc_give_the_same_rows(c1pq):
    import torch
    w, h, cb, idx = c1pq
    q = W.queries(w, batch=3, nq=24)
    ref = gpu_search(idx, q, w.nprobe, w.k)
    qd = torch.from_numpy(q).cuda()
    total = idx.info().index_bytes
    try:
        for frac in (0.4, 0.0, 1.0):
            say(f"C1-pq: device budget {frac:.1f} of the index")
            idx.set_device_budget(int(total * frac))
            got = gpu_search(idx, q, w.nprobe, w.k)
            assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])
        idx.set_device_budget(int(total * 0.3))
        idx.set_option("host_direct", 0)
        with pytest.raises(ivf.IvfError) as e:                   # the staged mode does not take code lists
            idx.search(qd, w.nprobe, w.k)
        assert e.value.code == -1
    finally:
        idx.set_option("host_direct", 1)
        idx.set_device_budget(2**62)
    idx.set_option("queue_min_mb", 0)
    st = torch.cuda.Stream()
    outs = [idx.search_queued(qd, w.nprobe, w.k, stream=st) for _ in range(7)]
    oi = torch.empty((24, w.k), dtype=torch.int64, device="cuda")
    os_ = torch.empty((24, w.k), dtype=torch.float32, device="cuda")
    idx.search_noalloc(qd, w.nprobe, w.k, oi, os_, stream=st)
    torch.cuda.synchronize()
    for ids, sc in outs + [(oi, os_)]:
        assert np.array_equal(ids.cpu().numpy(), ref[0]) and np.array_equal(sc.cpu().numpy(), ref[1])
    idx.set_option("queue_min_mb", 256)


CASES = [
    # name, n, d, M, nlist, empty lists, nq, nprobe, k
    ("m16_tiny", 300, 32, 16, 7, (2,), 9, 3, 7),
    ("m16_one_dim_per_code", 2000, 16, 16, 5, (), 6, 5, 20),
    ("m48_ragged", 5000, 96, 48, 13, (0, 12), 33, 4, 10),
    ("m128_largest_table", 3000, 256, 128, 6, (), 5, 3, 64),
    ("m32_k_above_candidates", 400, 64, 32, 9, (), 4, 2, 300),
    ("m16_one_list_many_queries", 3000, 48, 16, 1, (), 70, 1, 10),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_pq_edge_cases_match_oracle(case):
    name, n, d, M, nlist, empty, nq, nprobe, k = case
    rng = np.random.default_rng(sum(map(ord, name)))
    cen = rng.standard_normal((nlist, d)).astype(np.float32)
    x = rng.standard_normal((n, d)).astype(np.float32)
    cb = rng.standard_normal((M, 256, d // M)).astype(np.float32)
    sc = x.astype(np.float64) @ cen.astype(np.float64).T
    sc[:, list(empty)] = -np.inf
    lab = np.argmax(sc, axis=1)
    o = np.argsort(lab, kind="stable")
    x, lab = x[o], lab[o]
    off = np.zeros(nlist + 1, dtype=np.int64)
    np.cumsum(np.bincount(lab, minlength=nlist), out=off[1:])
    ids = rng.permutation(5 * n + 3)[:n].astype(np.int64)
    codes = W.pq_encode_host(x, cb)
    q = rng.standard_normal((nq, d)).astype(np.float32)
    idx = _upload(cen, codes, cb, ids, off)
    say(f"pq {name}: n={n} d={d} M={M} nlist={nlist} nq={nq} nprobe={nprobe} k={k}")
    got = gpu_search(idx, q, nprobe, k)
    xhat = PQ.decode(codes, cb)
    floor = float(np.linalg.norm(q, axis=1).max() * np.linalg.norm(xhat, axis=1).max())
    _check(cen, codes, cb, ids, off, q, nprobe, k, got, abs_floor=floor)
    idx.close()


def test_pq_argument_errors():
    idx = ivf.Index()
    cen = np.zeros((2, 32), dtype=np.float32)
    codes = np.zeros((4, 16), dtype=np.uint8)
    ids, off = np.arange(4, dtype=np.int64), np.array([0, 2, 4], dtype=np.int64)
    with pytest.raises(ivf.IvfError) as e:                       # no codebooks yet
        idx.upload(cen, codes, ids, off, dtype=ivf.IVF_PQ8)
    assert e.value.code == -1
    for m, code in ((8, -5), (144, -5)):                          # not a multiple of 16; above the largest table
        with pytest.raises(ivf.IvfError) as e:
            idx.set_pq_codebooks(np.zeros((m, 256, 2), dtype=np.float32))
        assert e.value.code == code
    idx.set_pq_codebooks(np.zeros((16, 256, 4), dtype=np.float32))    # d = 64, the index has d = 32
    with pytest.raises(ivf.IvfError) as e:
        idx.upload(cen, codes, ids, off, dtype=ivf.IVF_PQ8)
    assert e.value.code == -1
    idx.set_pq_codebooks(np.zeros((16, 256, 2), dtype=np.float32))
    idx.upload(cen, codes, ids, off, dtype=ivf.IVF_PQ8)
    with pytest.raises(ivf.IvfError):                             # the index holds codes of these codebooks
        idx.set_pq_codebooks(np.ones((16, 256, 2), dtype=np.float32))
    idx.close()


def test_c3_pq_full_size_matches_oracle():
    w = W.CONFIGS["C3-pq"]
    dw = DeviceWorkload(w)
    q = W.queries(w)
    say("C3-pq: search nq=64 nprobe=64 k=20")
    got = gpu_search(dw.index, q, w.nprobe, w.k)
    res = check_large(dw, q, w.nprobe, w.k, got)
    say(f"C3-pq ok: {res}")
    nblk = (np.diff(dw.off) + 63) // 64
    assert dw.index.info().index_bytes == int(nblk.sum()) * 64 * w.pq_m    # a sixteenth of the fp16 index
    dw.index.close()
