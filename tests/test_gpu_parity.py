"""GPU parity, small sizes: the HIP path (through the C ABI) against the CPU oracle,
element by element, on seeded inputs that span several 64-vector blocks, ragged tails,
empty lists, shared lists and the degenerate cases of the method."""
import zlib

import numpy as np
import pytest

from oracle import check as CK
from oracle import ivf_oracle as O
from paper_2504_15302_amd import ivf
from paper_2504_15302_amd import workloads as W
from tests.golden_util import load_basis_case
from tests.gpu_util import (check_against_oracle, gpu_search, say, upload_host_index)

pytestmark = pytest.mark.gpu


def _random_index(seed, n, d, nlist, storage, empty_lists=(), normalise=False):
    rng = np.random.default_rng(seed)
    cen = rng.standard_normal((nlist, d)).astype(np.float32)
    x = rng.standard_normal((n, d)).astype(np.float32)
    if normalise:
        cen /= np.linalg.norm(cen, axis=1, keepdims=True)
        x /= np.linalg.norm(x, axis=1, keepdims=True)
    sc = x.astype(np.float64) @ cen.astype(np.float64).T
    sc[:, list(empty_lists)] = -np.inf
    lab = np.argmax(sc, axis=1)
    order = np.argsort(lab, kind="stable")
    x, lab = x[order], lab[order]
    off = np.zeros(nlist + 1, dtype=np.int64)
    np.cumsum(np.bincount(lab, minlength=nlist), out=off[1:])
    ids = rng.permutation(7 * n + 13)[:n].astype(np.int64)          # unique, not contiguous
    vec = np.ascontiguousarray(x.astype(np.float16 if storage == "fp16" else np.float32))
    return cen, vec, ids, off


def _floor(q, vec):
    return float(np.linalg.norm(q, axis=1).max() * np.linalg.norm(vec.astype(np.float32), axis=1).max())


@pytest.fixture(scope="module")
def c1():
    w = W.CONFIGS["C1"]
    h = W.build_host_index(w)
    say("C1: uploading 100k x 384 fp32")
    return w, h, upload_host_index(h)


def test_c1_matches_oracle(c1):
    w, h, idx = c1
    q = W.queries(w)
    say("C1: search nq=16 nprobe=8 k=10")
    got = gpu_search(idx, q, w.nprobe, w.k)
    res = check_against_oracle(h.centroids, h.vectors, h.ids, h.offsets, q, w.nprobe, w.k, got, w.storage)
    say(f"C1 ok: {res}")
    st = idx.last_search_stats()
    o_probes = O.probe_select(O.coarse(q, h.centroids), w.nprobe)
    uniq = np.unique(o_probes)
    assert st.unique_lists == len(uniq) and st.pairs == w.nq * w.nprobe
    assert st.scanned_vectors == int(np.diff(h.offsets)[uniq].sum())
    assert st.scan_bytes == st.scanned_vectors * w.d * 4 and st.scan_bytes_streamed == 0


@pytest.mark.parametrize("k,nprobe,nq", [(1, 1, 1), (5, 3, 7), (100, 8, 16), (1024, 256, 3), (10, 300, 5)])
def test_c1_other_k_nprobe_nq(c1, k, nprobe, nq):
    w, h, idx = c1
    q = W.queries(w, batch=3, nq=nq)
    say(f"C1 variants: nq={nq} nprobe={nprobe} k={k}")
    got = gpu_search(idx, q, nprobe, k)
    check_against_oracle(h.centroids, h.vectors, h.ids, h.offsets, q, nprobe, k, got, w.storage)


def test_k_sweep_1_to_10(c1):
    """The paper's sensitivity study varies the number of retrieved chunks from 1 to 10
    (Section 6.5, "Number of Retrieval Chunks"): every k against the oracle, and each
    result the prefix of the next."""
    w, h, idx = c1
    q = W.queries(w, batch=5)
    prev = None
    for k in range(1, 11):
        say(f"C1: k={k}")
        got = gpu_search(idx, q, w.nprobe, k)
        check_against_oracle(h.centroids, h.vectors, h.ids, h.offsets, q, w.nprobe, k, got, w.storage)
        if prev is not None:
            assert np.array_equal(got[0][:, :k - 1], prev[0]) and np.array_equal(got[1][:, :k - 1], prev[1])
        prev = got


def test_rows_do_not_depend_on_the_batch(c1):
    w, h, idx = c1
    q = W.queries(w, batch=1)
    full = gpu_search(idx, q, w.nprobe, w.k)
    for r in (0, 5, 15):
        say(f"C1 batch independence: row {r} alone")
        one = gpu_search(idx, q[r:r + 1], w.nprobe, w.k)
        assert np.array_equal(one[0][0], full[0][r]) and np.array_equal(one[1][0], full[1][r])
    rev = gpu_search(idx, q[::-1].copy(), w.nprobe, w.k)
    assert np.array_equal(rev[0][::-1], full[0]) and np.array_equal(rev[1][::-1], full[1])


@pytest.mark.parametrize("storage", ["fp32", "fp16"])
def test_golden_basis_case_on_gpu(storage):
    g = load_basis_case(np.float16 if storage == "fp16" else np.float32)
    pad = 8 - g["d"]
    cen = np.pad(g["centroids"], ((0, 0), (0, pad)))
    vec = np.ascontiguousarray(np.pad(g["vectors"], ((0, 0), (0, pad))))
    idx = ivf.Index()
    idx.upload(np.ascontiguousarray(cen), vec, g["ids"], g["offsets"])
    for e in g["expects"]:
        q = np.pad(g["queries"][e["query"]], (0, pad))[None, :].astype(np.float32)
        say(f"golden basis case {storage}: {e['query']} nprobe={e['nprobe']} k={e['k']}")
        ids, scores, probes, coarse = gpu_search(idx, q, e["nprobe"], e["k"])
        assert probes[0].tolist() == e["probes"]
        assert ids[0].tolist() == e["ids"]                     # includes the id tie-break and the padding
        assert scores[0].tolist() == e["scores"]               # exact in binary
    idx.close()


CASES = [
    # name, n, d, nlist, storage, nq, nprobe, k, empty lists
    ("tiny_d8", 50, 8, 3, "fp32", 4, 2, 5, ()),
    ("one_vector", 1, 16, 1, "fp16", 2, 1, 3, ()),
    ("ragged_d72", 3000, 72, 7, "fp16", 9, 3, 10, ()),
    ("ragged_d40_fp32", 3000, 40, 7, "fp32", 9, 3, 10, ()),
    ("empty_lists", 2000, 32, 12, "fp32", 6, 12, 8, (0, 5, 11)),
    ("k_above_candidates", 300, 24, 6, "fp32", 5, 2, 400, ()),
    ("all_lists", 5000, 64, 33, "fp16", 8, 33, 20, ()),
    ("many_blocks", 40000, 128, 5, "fp16", 6, 2, 50, ()),
    ("wide_d1024", 1500, 1024, 4, "fp32", 3, 2, 10, ()),
    # the documented maxima: d = 4096; k = nprobe = 1024; nq = 65535
    ("max_d4096", 600, 4096, 3, "fp16", 3, 2, 10, ()),
    ("max_k_and_nprobe_1024", 40000, 16, 1100, "fp32", 3, 1024, 1024, (7,)),
    ("max_nq_65535", 200, 8, 2, "fp32", 65535, 1, 1, ()),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_edge_cases_match_oracle(case):
    name, n, d, nlist, storage, nq, nprobe, k, empty = case
    cen, vec, ids, off = _random_index(zlib.crc32(name.encode()) % 1000, n, d, nlist, storage, empty)
    rng = np.random.default_rng(99)
    q = rng.standard_normal((nq, d)).astype(np.float32)
    idx = ivf.Index()
    idx.upload(cen, vec, ids, off)
    say(f"edge case {name}")
    got = gpu_search(idx, q, nprobe, k)
    check_against_oracle(cen, vec, ids, off, q, nprobe, k, got, storage, abs_floor=_floor(q, vec))
    idx.close()


def test_many_queries_share_one_list():
    """More than kQB queries on the same list: several query groups per block."""
    cen, vec, ids, off = _random_index(5, 6000, 64, 4, "fp16", normalise=True)
    rng = np.random.default_rng(1)
    base = cen[2]
    q = (base[None, :] + 0.05 * rng.standard_normal((23, 64))).astype(np.float32)
    idx = ivf.Index()
    idx.upload(cen, vec, ids, off)
    say("23 queries probing the same lists")
    got = gpu_search(idx, q, 2, 15)
    check_against_oracle(cen, vec, ids, off, q, 2, 15, got, "fp16")
    st = idx.last_search_stats()
    assert st.unique_lists <= 4 and st.pairs == 46
    idx.close()


def test_skewed_batch_sixteen_queries_per_list(c1):
    """A batch whose 128 queries come from 8 mixture components: every home list is probed
    by about 16 queries (the other probes of a query depend on its noise and are shared
    less), so its blocks are shared by several groups of four queries."""
    w, h, idx = c1
    q = W.queries(w, batch=9, nq=128, components=8)
    say("C1 skewed: nq=128 from 8 components, nprobe=8 k=10")
    got = gpu_search(idx, q, w.nprobe, w.k)
    check_against_oracle(h.centroids, h.vectors, h.ids, h.offsets, q, w.nprobe, w.k, got, w.storage)
    st = idx.last_search_stats()
    probes = got[2]
    cnt = np.bincount(probes.ravel(), minlength=w.nlist)
    nblk = (np.diff(h.offsets) + 63) // 64
    assert st.pairs == 128 * w.nprobe and st.unique_lists == int((cnt > 0).sum())
    assert (cnt >= 12).sum() >= 8 and st.pairs / st.unique_lists >= 3      # really skewed
    assert st.scan_items == int((nblk * ((cnt + 3) // 4)).sum())   # one item per block and group of 4 queries
    # the same rows when each query is searched in a batch of its own component only
    sub = q[::16]
    one = gpu_search(idx, sub, w.nprobe, w.k)
    assert np.array_equal(one[0], got[0][::16]) and np.array_equal(one[1], got[1][::16])
    # near copies of 8 queries: every probed list is shared by about 16 queries
    q = W.queries(w, batch=9, nq=128, components=8, tight=True)
    say("C1 skewed, tight: every probed list shared by ~16 queries")
    got = gpu_search(idx, q, w.nprobe, w.k)
    check_against_oracle(h.centroids, h.vectors, h.ids, h.offsets, q, w.nprobe, w.k, got, w.storage)
    st = idx.last_search_stats()
    assert st.pairs / st.unique_lists >= 10


@pytest.mark.parametrize("nq", [33, 64, 65, 129, 300])
def test_batch_sizes_across_the_coarse_kernel_tilings(c1, nq):
    """nq <= 32, <= 64 and above take different query-tile shapes in the coarse kernel;
    above 128 the grid gets a second row of workgroups."""
    w, h, idx = c1
    q = W.queries(w, batch=7, nq=nq)
    say(f"C1 nq={nq} nprobe=4 k=7")
    got = gpu_search(idx, q, 4, 7)
    check_against_oracle(h.centroids, h.vectors, h.ids, h.offsets, q, 4, 7, got, w.storage)


@pytest.mark.parametrize("seed", range(4))
def test_random_shapes_match_oracle(seed):
    """Seeded random shapes: list count, dimension, storage type, batch, nprobe and k."""
    rng = np.random.default_rng(1000 + seed)
    nlist = int(rng.integers(1, 90))
    d = 8 * int(rng.integers(1, 40))
    n = int(rng.integers(1, 20000))
    storage = "fp16" if rng.integers(2) else "fp32"
    nq = int(rng.integers(1, 70))
    nprobe = int(rng.integers(1, nlist + 3))
    k = int(rng.integers(1, 300))
    cen, vec, ids, off = _random_index(seed, n, d, nlist, storage)
    q = rng.standard_normal((nq, d)).astype(np.float32)
    idx = ivf.Index()
    idx.upload(cen, vec, ids, off)
    idx.set_option("scan_prune", 2)
    say(f"random case {seed}: n={n} d={d} nlist={nlist} {storage} nq={nq} nprobe={nprobe} k={k}")
    got = gpu_search(idx, q, nprobe, k)
    check_against_oracle(cen, vec, ids, off, q, nprobe, k, got, storage, abs_floor=_floor(q, vec))
    idx.close()


def test_exact_ties_go_to_the_smaller_id():
    d = 16
    rng = np.random.default_rng(8)
    v = rng.standard_normal(d).astype(np.float32)
    rows = [v, v, v * 0.5, v, v * 0.25, v]
    vec = np.stack(rows).astype(np.float32)
    ids = np.array([90, 40, 10, 70, 5, 41], dtype=np.int64)
    off = np.array([0, 3, 6], dtype=np.int64)
    cen = np.stack([v, v * 0.9]).astype(np.float32)
    idx = ivf.Index()
    idx.upload(cen, vec, ids, off)
    say("exact score ties across two lists")
    gi, gs, _, _ = gpu_search(idx, v[None, :], 2, 6)
    oi, os_, _, _ = O.search(cen, vec, ids, off, v[None, :], 2, 6)
    assert gi[0].tolist() == oi[0].tolist() == [40, 41, 70, 90, 10, 5]
    assert gs[0, 0] == gs[0, 3]
    idx.close()


def test_upload_in_pieces_and_from_device_memory_equals_one_shot(c1):
    import torch
    w, h, idx = c1
    q = W.queries(w, batch=2)
    ref = gpu_search(idx, q, w.nprobe, w.k)
    say("C1 uploaded in pieces from device memory")
    idx2 = ivf.Index()
    idx2.upload_begin(h.centroids, w.n, ivf.IVF_FP32, h.offsets)
    cuts = [0, 1, 64, 65, 200, 256]
    for a, b in zip(cuts[:-1], cuts[1:]):
        r0, r1 = int(h.offsets[a]), int(h.offsets[b])
        vd = torch.from_numpy(h.vectors[r0:r1]).cuda()
        idd = torch.from_numpy(h.ids[r0:r1]).cuda()
        idx2.upload_lists(a, b, vd, idd)
    idx2.upload_end()
    got = gpu_search(idx2, q, w.nprobe, w.k)
    assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])
    for l in (0, 17, 255):
        vec, ids = idx2.read_list(l, w.d, ivf.IVF_FP32)
        assert np.array_equal(vec, h.vectors[h.offsets[l]:h.offsets[l + 1]])
        assert np.array_equal(ids, h.ids[h.offsets[l]:h.offsets[l + 1]])
    idx2.close()


def test_results_do_not_depend_on_placement(c1):
    w, h, idx = c1
    q = W.queries(w, batch=4)
    ref = gpu_search(idx, q, w.nprobe, w.k)
    total = idx.info().index_bytes
    for frac in (0.25, 0.0, 0.6, 1.0):
        say(f"C1 device budget {frac:.2f} of the index")
        idx.set_device_budget(int(total * frac))
        info = idx.info()
        assert info.device_list_bytes <= int(total * frac)
        assert info.device_list_bytes + info.host_list_bytes == total
        got = gpu_search(idx, q, w.nprobe, w.k)
        assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])
        st = idx.last_search_stats()
        assert st.scan_bytes_resident + st.scan_bytes_streamed == st.scan_bytes
        if frac == 0.0:
            assert st.scan_bytes_resident == 0 and info.resident_lists == 0
        for l in (3, 100):
            vec, ids = idx.read_list(l, w.d, ivf.IVF_FP32)
            assert np.array_equal(vec, h.vectors[h.offsets[l]:h.offsets[l + 1]])
    check_against_oracle(h.centroids, h.vectors, h.ids, h.offsets, q, w.nprobe, w.k, ref, w.storage)
    # the same with host-resident lists copied to staging buffers with hipMemcpyAsync on
    # the side stream (default: the scan reads them in place from pinned host memory)
    try:
        idx.set_option("host_direct", 0)
        for frac, stage_mb, nstage in ((0.3, 64, 3), (0.0, 1, 2), (0.5, 2, 4)):
            idx.set_option("stage_mb", stage_mb)
            idx.set_option("nstage", nstage)
            idx.set_device_budget(int(total * frac))
            for rep in range(2):
                say(f"C1 device budget {frac:.2f}, staged copies ({nstage} x {stage_mb} MiB), run {rep}")
                got = gpu_search(idx, q, w.nprobe, w.k)
                assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])
            st = idx.last_search_stats()
            assert st.scan_bytes_streamed > 0 and st.scan_bytes_resident + st.scan_bytes_streamed == st.scan_bytes
    finally:
        idx.set_option("host_direct", 1)
        idx.set_option("stage_mb", 64)
        idx.set_option("nstage", 3)
        idx.set_device_budget(2**62)


def test_budget_changes_move_only_the_difference_and_give_memory_back(c1):
    """Repeated budget changes between batches (the paper changes the number of resident
    partitions at run time, Sections 4.2 and 5): only lists that change tier cross PCIe,
    the HBM pool shrinks with the budget, results never change."""
    w, h, idx = c1
    q = W.queries(w, batch=8)
    ref = gpu_search(idx, q, w.nprobe, w.k)
    lens = np.diff(h.offsets)
    nblk = (lens + 63) // 64
    bb = 64 * w.d * 4
    order = np.lexsort((np.arange(w.nlist), -lens))
    total = int(nblk.sum()) * bb
    seg = 64 << 20                                   # C1 is smaller than 16 segments of 64 MiB

    def resident_set(budget):
        used, keep = 0, set()
        for l in order:
            b = int(nblk[l]) * bb
            if used + b > budget:
                break
            used += b
            keep.add(int(l))
        return keep

    cur = set(range(w.nlist))
    try:
        for frac in (0.25, 0.30, 0.10, 0.0, 0.5, 1.0):
            budget = int(total * frac)
            want = resident_set(budget)
            say(f"C1 budget -> {frac:.2f}: {len(want)} lists resident")
            idx.set_device_budget(budget)
            info = idx.info()
            assert info.resident_lists == len(want)
            out_b = sum(int(nblk[l]) * bb for l in cur - want)
            in_b = sum(int(nblk[l]) * bb for l in want - cur)
            assert info.moved_d2h_bytes == out_b and info.moved_h2d_bytes == in_b
            res_b = sum(int(nblk[l]) * bb for l in want)
            assert info.device_list_bytes == res_b and info.host_list_bytes == total - res_b
            assert res_b <= info.device_pool_bytes <= res_b + 2 * seg
            assert total - res_b <= info.host_pool_bytes <= total - res_b + 2 * seg
            got = gpu_search(idx, q, w.nprobe, w.k)
            assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])
            for l in (0, 77, 255):
                vec, ids = idx.read_list(l, w.d, ivf.IVF_FP32)
                assert np.array_equal(vec, h.vectors[h.offsets[l]:h.offsets[l + 1]])
                assert np.array_equal(ids, h.ids[h.offsets[l]:h.offsets[l + 1]])
            cur = want
    finally:
        idx.set_device_budget(2**62)


def test_most_probed_lists_stay_resident_under_the_hot_policy(c1):
    w, h, _ = c1
    idx = upload_host_index(h)                      # fresh probe counts
    q = W.queries(w, batch=9)
    ref = gpu_search(idx, q, w.nprobe, w.k)
    probed = np.unique(ref[2])
    nblk = (np.diff(h.offsets) + 63) // 64
    bb = 64 * w.d * 4
    budget = int(sum(int(nblk[l]) for l in probed)) * bb
    say("C1 budget = size of the probed lists, ranked by length")
    idx.set_device_budget(budget)
    got = gpu_search(idx, q, w.nprobe, w.k)
    assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])
    assert idx.last_search_stats().scan_bytes_streamed > 0
    say("C1 same budget, ranked by probe count")
    idx.set_option("residency_policy", 1)
    idx.set_device_budget(budget)
    got = gpu_search(idx, q, w.nprobe, w.k)
    assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])
    st = idx.last_search_stats()
    assert st.scan_bytes_streamed == 0 and idx.info().resident_lists == len(probed)
    idx.close()


def test_fused_and_separate_regrouping_agree(c1):
    w, h, idx = c1
    try:
        for nq, nprobe, k in ((16, 8, 10), (130, 15, 7), (3, 256, 100), (250, 8, 5)):
            q = W.queries(w, batch=51, nq=nq)
            idx.set_option("regroup_fused", 1)
            a = gpu_search(idx, q, nprobe, k)
            sa = idx.last_search_stats()
            idx.set_option("regroup_fused", 0)
            b = gpu_search(idx, q, nprobe, k)
            sb = idx.last_search_stats()
            assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]), (nq, nprobe, k)
            for f in ("unique_lists", "pairs", "scanned_vectors", "scan_bytes", "scan_bytes_resident", "scan_items"):
                assert getattr(sa, f) == getattr(sb, f), f
        total = idx.info().index_bytes
        idx.set_device_budget(int(total * 0.4))             # host-resident lists in the plan
        q = W.queries(w, batch=52)
        idx.set_option("regroup_fused", 1)
        a = gpu_search(idx, q, w.nprobe, w.k)
        idx.set_option("regroup_fused", 0)
        b = gpu_search(idx, q, w.nprobe, w.k)
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    finally:
        idx.set_option("regroup_fused", 1)
        idx.set_device_budget(2**62)


def test_selection_workgroup_sizes_agree(c1):
    w, h, idx = c1
    try:
        for nq, nprobe, k in ((16, 8, 10), (5, 200, 1000), (40, 1, 1)):
            q = W.queries(w, batch=50, nq=nq)
            idx.set_option("sel_threads", 0)
            ref = gpu_search(idx, q, nprobe, k)
            for t in (256, 1024):
                idx.set_option("sel_threads", t)
                got = gpu_search(idx, q, nprobe, k)
                assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1]) and np.array_equal(got[2], ref[2]), (t, nq, nprobe, k)
    finally:
        idx.set_option("sel_threads", 0)


def test_scan_launch_options_agree(c1):
    w, h, idx = c1
    q = W.queries(w, batch=5)
    ref = gpu_search(idx, q, w.nprobe, w.k)
    try:
        # register-buffer width and workgroup size never change the order of the additions;
        # the number of wavefronts per block does (last bits of the scores only)
        for split, unroll, waves in [(0, 8, 4), (0, 16, 4), (1, 8, 4), (1, 16, 4), (1, 16, 1), (1, 16, 2),
                                     (1, 8, 8), (2, 16, 4), (2, 8, 4), (4, 8, 4)]:
            say(f"C1 scan_split={split} scan_unroll={unroll} scan_waves={waves}")
            idx.set_option("scan_split", split)
            idx.set_option("scan_unroll", unroll)
            idx.set_option("scan_waves", waves)
            got = gpu_search(idx, q, w.nprobe, w.k)
            assert np.array_equal(got[0], ref[0])
            if split in (0, 2):                      # C1's blocks (96 KiB) take two wavefronts by default
                assert np.array_equal(got[1], ref[1])
            else:
                assert np.allclose(got[1], ref[1], rtol=1e-6)
    finally:
        idx.set_option("scan_split", 0)
        idx.set_option("scan_unroll", 16)
        idx.set_option("scan_waves", 4)


SPLIT_CASES = [
    # name, n, d, nlist, storage, nq, nprobe, k: dimensions whose chunks split evenly, unevenly and not at all
    ("split_d768_fp16", 6000, 768, 9, "fp16", 11, 3, 20),
    ("split_d768_fp32", 4000, 768, 7, "fp32", 6, 3, 100),
    ("split_d8", 900, 8, 5, "fp16", 7, 2, 10),
    ("split_d40_fp32", 3000, 40, 7, "fp32", 9, 3, 10),
    ("split_d200_fp16", 3000, 200, 6, "fp16", 23, 6, 64),
]


@pytest.mark.parametrize("case", SPLIT_CASES, ids=[c[0] for c in SPLIT_CASES])
def test_scan_with_several_wavefronts_per_block_matches_oracle(case):
    """scan_split = 2 | 4: the dimensions of a block are shared out over wavefronts and the
    partial sums added in LDS (another order of additions than one wavefront per block:
    compared with the oracle, not bit for bit with the unsplit scan), with and without
    store pruning, in both host-list modes."""
    name, n, d, nlist, storage, nq, nprobe, k = case
    cen, vec, ids, off = _random_index(zlib.crc32(name.encode()) % 1000, n, d, nlist, storage, normalise=True)
    rng = np.random.default_rng(17)
    q = rng.standard_normal((nq, d)).astype(np.float32)
    q[:nq // 2] = cen[rng.integers(0, nlist, nq // 2)] + 0.1 * q[:nq // 2]      # several queries per list
    idx = ivf.Index()
    idx.upload(cen, vec, ids, off)
    for split in (2, 4):
        idx.set_option("scan_split", split)
        for prune in (1, 2):
            idx.set_option("scan_prune", prune)
            say(f"{name}: scan_split={split} scan_prune={prune}")
            got = gpu_search(idx, q, nprobe, k)
            check_against_oracle(cen, vec, ids, off, q, nprobe, k, got, storage, abs_floor=_floor(q, vec))
        idx.set_device_budget(idx.info().index_bytes // 2)
        part = gpu_search(idx, q, nprobe, k)
        assert np.array_equal(part[0], got[0]) and np.array_equal(part[1], got[1])
        idx.set_option("host_direct", 0)
        staged = gpu_search(idx, q, nprobe, k)
        assert np.array_equal(staged[0], got[0]) and np.array_equal(staged[1], got[1])
        idx.set_option("host_direct", 1)
        idx.set_device_budget(2**62)
    idx.close()


@pytest.mark.parametrize("k", [1, 10, 64, 65, 100, 128, 129])
def test_store_pruning_in_the_scan_does_not_change_results(c1, k):
    """The scan skips storing blocks below its running bound of the k-th best score
    (one-block bound up to k=64, two-block bound up to k=128, none above)."""
    w, h, idx = c1
    q = W.queries(w, batch=6)
    try:
        idx.set_option("scan_prune", 0)
        say(f"C1 k={k} without store pruning")
        ref = gpu_search(idx, q, 16, k)
        idx.set_option("scan_prune", 2)       # forced: C1's plan is below the size where it switches on
        for rep in range(2):
            say(f"C1 k={k} with store pruning, run {rep}")
            got = gpu_search(idx, q, 16, k)
            assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])
    finally:
        idx.set_option("scan_prune", 1)
    check_against_oracle(h.centroids, h.vectors, h.ids, h.offsets, q, 16, k, ref, w.storage)


def test_error_paths_on_the_gpu(c1):
    import torch
    w, h, idx = c1
    q = torch.zeros((2, w.d), device="cuda")
    oi = torch.empty((2, 4), dtype=torch.int64, device="cuda")
    os_ = torch.empty((2, 4), dtype=torch.float32, device="cuda")
    assert idx.search_raw(None, 2, 1, 4, oi.data_ptr(), os_.data_ptr()) == -1
    assert idx.search_raw(q.data_ptr(), 2, 0, 4, oi.data_ptr(), os_.data_ptr()) == -1
    assert idx.search_raw(q.data_ptr(), 2, 1, 0, oi.data_ptr(), os_.data_ptr()) == -1
    assert idx.search_raw(q.data_ptr(), 2, 1, 5000, oi.data_ptr(), os_.data_ptr()) == -5
    assert idx.search_raw(q.data_ptr(), -1, 1, 4, oi.data_ptr(), os_.data_ptr()) == -1
    assert idx.search_raw(q.data_ptr(), 0, 1, 4, oi.data_ptr(), os_.data_ptr()) == 0
    with pytest.raises(ivf.IvfError):
        idx.set_device_budget(-1)
    with pytest.raises(ivf.IvfError):
        idx.set_option("no_such_option", 1)
    empty = ivf.Index()
    assert empty.search_raw(q.data_ptr(), 2, 1, 4, oi.data_ptr(), os_.data_ptr()) == -1
    with pytest.raises(ivf.IvfError):      # d not a multiple of 8
        empty.upload(np.zeros((2, 12), np.float32), np.zeros((4, 12), np.float32),
                     np.arange(4, dtype=np.int64), np.array([0, 2, 4], dtype=np.int64))
    with pytest.raises(ivf.IvfError):      # offsets do not end at n
        empty.upload(np.zeros((2, 16), np.float32), np.zeros((4, 16), np.float32),
                     np.arange(4, dtype=np.int64), np.array([0, 2, 3], dtype=np.int64))
    empty.close()
    # the index still works after the failed calls
    got = gpu_search(idx, W.queries(w), w.nprobe, w.k)
    check_against_oracle(h.centroids, h.vectors, h.ids, h.offsets, W.queries(w), w.nprobe, w.k, got, w.storage)


def test_search_can_be_captured_in_a_hip_graph_and_replayed(c1):
    """After one eager call with the same shapes (scratch is allocated on first use) a
    search records only kernel launches on the caller's stream — no allocation, no host
    synchronisation, no memset node — so a caller may capture it in a HIP graph.  Replays,
    with eager work and synchronisations in between, are checked against eager results."""
    import torch
    w, h, idx = c1
    nq = 16
    batches = [W.queries(w, batch=30 + b, nq=nq) for b in range(4)]
    refs = [gpu_search(idx, q, w.nprobe, w.k) for q in batches]
    q_static = torch.from_numpy(batches[0]).cuda()
    out_ids = torch.empty((nq, w.k), dtype=torch.int64, device="cuda")
    out_scores = torch.empty((nq, w.k), dtype=torch.float32, device="cuda")
    idx.search(q_static, w.nprobe, w.k, out_ids, out_scores)          # warm-up with these shapes
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    say("C1: capturing one search in a HIP graph")
    with torch.cuda.graph(g):
        idx.search(q_static, w.nprobe, w.k, out_ids, out_scores)
    for rep in range(3):
        for b, q in enumerate(batches):
            q_static.copy_(torch.from_numpy(q).cuda())
            out_ids.fill_(-7)
            g.replay()
            torch.cuda.synchronize()
            assert np.array_equal(out_ids.cpu().numpy(), refs[b][0]), f"replay {rep}, batch {b}"
            assert np.array_equal(out_scores.cpu().numpy(), refs[b][1])
            eager = gpu_search(idx, batches[(b + 1) % 4], w.nprobe, w.k)   # the library's own eager work in between
            assert np.array_equal(eager[0], refs[(b + 1) % 4][0])
    del g


def test_plain_c_consumer_of_the_abi():
    """examples/search_demo.c, built by the package's build step: upload from host arrays,
    half of the index in pinned host memory, search, its own brute-force check."""
    import subprocess
    from paper_2504_15302_amd import build
    say("running the C demo")
    r = subprocess.run([build.DEMO], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout + r.stderr


def test_two_indexes_on_two_streams_and_two_threads_do_not_interfere():
    """Different indexes share nothing: searches on two indexes queued alternately on two
    streams, and issued from two host threads at once, return what each index returns alone."""
    import threading
    import torch
    a = _random_index(21, 9000, 64, 12, "fp16", normalise=True)
    b = _random_index(22, 7000, 96, 9, "fp32")
    rng = np.random.default_rng(5)
    qa = rng.standard_normal((20, 64)).astype(np.float32)
    qb = rng.standard_normal((33, 96)).astype(np.float32)
    ia, ib = ivf.Index(), ivf.Index()
    ia.upload(*a)
    ib.upload(*b)
    ra = gpu_search(ia, qa, 4, 10)
    rb = gpu_search(ib, qb, 3, 17)
    check_against_oracle(*a, qa, 4, 10, ra, "fp16", abs_floor=_floor(qa, a[1]))
    check_against_oracle(*b, qb, 3, 17, rb, "fp32", abs_floor=_floor(qb, b[1]))
    say("two indexes, two streams, searches queued alternately")
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    da, db = torch.from_numpy(qa).cuda(), torch.from_numpy(qb).cuda()
    torch.cuda.synchronize()
    outs = []
    for rep in range(20):
        outs.append(("a", ia.search(da, 4, 10, stream=sa)))
        outs.append(("b", ib.search(db, 3, 17, stream=sb)))
    torch.cuda.synchronize()
    for which, (ids, sc) in outs:
        ref = ra if which == "a" else rb
        assert np.array_equal(ids.cpu().numpy(), ref[0]) and np.array_equal(sc.cpu().numpy(), ref[1])
    say("two indexes, two host threads")
    errors = []

    def worker(idx, dq, nprobe, k, ref, stream):
        try:
            for rep in range(50):
                ids, sc = idx.search(dq, nprobe, k, stream=stream)
                stream.synchronize()
                if not (np.array_equal(ids.cpu().numpy(), ref[0]) and np.array_equal(sc.cpu().numpy(), ref[1])):
                    errors.append(f"mismatch at repetition {rep}")
                    return
        except Exception as e:                      # noqa: BLE001
            errors.append(repr(e))

    th = [threading.Thread(target=worker, args=(ia, da, 4, 10, ra, sa)),
          threading.Thread(target=worker, args=(ib, db, 3, 17, rb, sb))]
    for t in th:
        t.start()
    for t in th:
        t.join(timeout=120)
        assert not t.is_alive()
    assert not errors, errors
    ia.close()
    ib.close()


def test_timing_levels(c1):
    w, h, idx = c1
    q = W.queries(w, batch=40)
    try:
        idx.set_timing(1)
        gpu_search(idx, q, w.nprobe, w.k)
        ms = idx.stage_ms(0)
        assert all(ms[s] > 0 for s in ("coarse", "probe", "regroup", "scan", "select"))
        assert abs(ms["total"] - sum(ms[s] for s in ivf.STAGES[:-1])) < 0.05 * ms["total"] + 1e-3
        idx.set_timing(2)                                   # the scan and streaming stages only
        gpu_search(idx, q, w.nprobe, w.k)
        ms = idx.stage_ms(0)
        assert ms["scan"] > 0 and ms["coarse"] == 0 and ms["select"] == 0
        assert abs(ms["total"] - ms["scan"] - ms["stream"]) < 0.05 * ms["total"] + 1e-3
        with pytest.raises(ivf.IvfError):
            idx.set_timing(3)
        idx.set_timing(0)
        gpu_search(idx, q, w.nprobe, w.k)
        with pytest.raises(ivf.IvfError):
            idx.stage_ms(0)                                 # nothing was timed
    finally:
        idx.set_timing(0)
