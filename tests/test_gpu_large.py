"""GPU parity at the benchmark's full sizes (C2..C5), in the launch configuration
bench.py times.  The index is generated on the device and handed to the library in
pieces; the oracle sees only the probed lists, regenerated from the seeded recipe and
copied to the host.  Every configuration is checked on every query row."""
import numpy as np
import pytest

from oracle import ivf_oracle as O
from paper_2504_15302_amd import ivf
from paper_2504_15302_amd import workloads as W
from tests.gpu_util import DeviceWorkload, check_large, gpu_search, say

pytestmark = pytest.mark.gpu


def _check_assignment_sample(dw, nsample_lists=24, nvec=10000):
    """The list a vector was generated for is its arg-max inner-product centroid (fp64, on a
    random sample: every centroid is streamed once per sampled vector, which bounds the
    sample at the largest index)."""
    rng = np.random.default_rng(0)
    lists = rng.choice(dw.w.nlist, size=nsample_lists, replace=False)
    vec, ids, coff, cmap = dw.host_lists(lists)
    take = rng.choice(vec.shape[0], size=min(nvec, vec.shape[0]), replace=False)
    lab, _ = O.assign(vec[take], dw.cen)
    truth = np.empty(vec.shape[0], dtype=np.int32)
    for l, c in cmap.items():
        truth[coff[c]:coff[c + 1]] = l
    assert np.array_equal(lab, truth[take])


def _check_readback(dw, lists):
    vec, ids, coff, cmap = dw.host_lists(lists)
    dt = ivf.IVF_FP16 if dw.w.storage == "fp16" else ivf.IVF_FP32
    for l in lists:
        v, i = dw.index.read_list(int(l), dw.w.d, dt)
        c = cmap[int(l)]
        assert np.array_equal(v, vec[coff[c]:coff[c + 1]]) and np.array_equal(i, ids[coff[c]:coff[c + 1]])


def test_c2_full_size_matches_oracle():
    w = W.CONFIGS["C2"]
    dw = DeviceWorkload(w)
    q = W.queries(w)
    say("C2: search nq=32 nprobe=32 k=10")
    got = gpu_search(dw.index, q, w.nprobe, w.k)
    res = check_large(dw, q, w.nprobe, w.k, got)
    say(f"C2 ok: {res}")
    _check_assignment_sample(dw)
    _check_readback(dw, [0, 1234, w.nlist - 1])
    st = dw.index.last_search_stats()
    assert st.pairs == w.nq * w.nprobe and st.scan_bytes == st.scanned_vectors * w.d * 4
    dw.index.close()


@pytest.fixture(scope="module")
def c3():
    dw = DeviceWorkload(W.CONFIGS["C3"])
    yield dw
    dw.index.close()


def test_c3_full_size_matches_oracle(c3):
    w = c3.w
    q = W.queries(w)
    say("C3: search nq=64 nprobe=64 k=20")
    got = gpu_search(c3.index, q, w.nprobe, w.k)
    res = check_large(c3, q, w.nprobe, w.k, got)
    say(f"C3 ok: {res}")
    _check_assignment_sample(c3, nvec=4000)
    _check_readback(c3, [5, 9000])


def test_c4_offloaded_placement_matches_oracle_and_c3(c3):
    """Same index and queries as C3 (its first 8), with only the 25 % longest lists
    (by count, ranked by length then list number) resident in HBM."""
    w = W.CONFIGS["C4"]
    q = W.queries(w)
    assert np.array_equal(q, W.queries(W.CONFIGS["C3"])[:w.nq])
    say("C4: reference search with everything resident")
    ref = gpu_search(c3.index, q, w.nprobe, w.k)
    lens = np.diff(c3.off)
    order = np.lexsort((np.arange(w.nlist), -lens))
    keep = order[: int(w.nlist * w.resident_list_frac)]
    nblk = (lens + 63) // 64
    budget = int(nblk[keep].sum()) * 64 * w.d * 2
    say(f"C4: device budget {budget / 2**30:.2f} GiB -> moving lists to pinned host memory")
    c3.index.set_device_budget(budget)
    info = c3.index.info()
    assert info.resident_lists == len(keep) and info.device_list_bytes == budget
    say("C4: offloaded search nq=8 nprobe=64 k=20")
    got = gpu_search(c3.index, q, w.nprobe, w.k)
    assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])
    res = check_large(c3, q, w.nprobe, w.k, got)
    st = c3.index.last_search_stats()
    assert st.scan_bytes_streamed > 0 and st.scan_bytes_resident + st.scan_bytes_streamed == st.scan_bytes
    say(f"C4 ok: {res}; streamed {st.scan_bytes_streamed / 1e6:.0f} MB, resident {st.scan_bytes_resident / 1e6:.0f} MB")
    _check_readback(c3, [int(order[0]), int(order[-1])])
    # the staged variant: hipMemcpyAsync to staging buffers on the side stream, two batches
    # through the same buffers
    c3.index.set_option("host_direct", 0)
    try:
        say("C4: offloaded search through staging copies")
        got_s = gpu_search(c3.index, q, w.nprobe, w.k)
        assert np.array_equal(got_s[0], ref[0]) and np.array_equal(got_s[1], ref[1])
        q2 = W.queries(W.CONFIGS["C3"], batch=1)[:w.nq]
        got2 = gpu_search(c3.index, q2, w.nprobe, w.k)
        check_large(c3, q2, w.nprobe, w.k, got2)
    finally:
        c3.index.set_option("host_direct", 1)
    say("C4: back to fully resident")
    c3.index.set_device_budget(2**62)
    got3 = gpu_search(c3.index, q, w.nprobe, w.k)
    assert np.array_equal(got3[0], ref[0]) and np.array_equal(got3[1], ref[1])


def test_c3_worker_serves_requests_while_the_budget_changes(c3):
    """The pipeline's retrieval half at full size: client threads keep a worker busy while
    its index goes from fully resident to a quarter of the lists and back (23 GB each way
    on streams of their own); every request gets the rows of a direct search."""
    import threading
    import time
    w = c3.w
    q = W.queries(w, batch=2)                                  # 64 queries
    ref = gpu_search(c3.index, q, w.nprobe, w.k)
    check_large(c3, q, w.nprobe, w.k, ref, rows=[0, 63])
    lens = np.diff(c3.off)
    order = np.lexsort((np.arange(w.nlist), -lens))
    keep = order[: w.nlist // 4]
    quarter = int(((lens[keep] + 63) // 64).sum()) * 64 * w.d * 2
    wk = ivf.Worker(c3.index, w.nprobe, w.k, 16)
    results, stop = {}, threading.Event()

    def client(c):
        r = 0
        while not stop.is_set():
            i = (c * 7 + r) % 64
            got = wk.wait(wk.submit(q[i]))
            results[(c, r)] = (i, got)
            r += 1

    try:
        th = [threading.Thread(target=client, args=(c,)) for c in range(4)]
        for t in th:
            t.start()
        seen = []
        for target, want in ((quarter, len(keep)), (2**62, w.nlist)):
            say(f"C3 worker: budget change to {want} resident lists under load")
            wk.set_device_budget(target)
            t0 = time.time()
            while time.time() - t0 < 120:
                st = wk.stats()
                seen.append(st.resident_lists)
                if not st.budget_busy and st.resident_lists == want:
                    break
                time.sleep(0.02)
            st = wk.stats()
            assert st.budget_busy == 0 and st.budget_error == 0 and st.resident_lists == want, (st.resident_lists, want)
        stop.set()
        for t in th:
            t.join(timeout=60)
            assert not t.is_alive()
    finally:
        stop.set()
        wk.stop()
    assert len(results) > 20
    for (c, r), (i, got) in results.items():
        assert np.array_equal(got[0], ref[0][i]) and np.array_equal(got[1], ref[1][i]), f"client {c} request {r}"
    assert any(len(keep) < s < w.nlist for s in seen)          # the change was seen half-way
    say(f"C3 worker: {len(results)} requests answered during the two changes")
    assert c3.index.info().resident_lists == w.nlist


def test_c5_full_size_every_row_matches_oracle():
    w = W.CONFIGS["C5"]
    dw = DeviceWorkload(w, groups_per_chunk=32)
    q = W.queries(w)
    say("C5: search nq=128 nprobe=128 k=100")
    got = gpu_search(dw.index, q, w.nprobe, w.k)
    res = check_large(dw, q, w.nprobe, w.k, got)
    assert res["queries"] == w.nq
    say(f"C5 ok on all {w.nq} rows: {res}")
    # the launch configuration that bench.py times: searches queued back to back on a stream
    # of the caller's, stages of neighbours overlapping; rows are those of the plain search
    import torch
    say("C5: six queued searches over two batches")
    q2 = W.queries(w, batch=1)
    got2 = gpu_search(dw.index, q2, w.nprobe, w.k)
    qd = [torch.from_numpy(q).cuda(), torch.from_numpy(q2).cuda()]
    st = torch.cuda.Stream()
    torch.cuda.synchronize()
    outs = [dw.index.search_queued(qd[i % 2], w.nprobe, w.k, stream=st) for i in range(6)]
    st.synchronize()
    for i, (ids, sc) in enumerate(outs):
        ref = got if i % 2 == 0 else got2
        assert np.array_equal(ids.cpu().numpy(), ref[0]) and np.array_equal(sc.cpu().numpy(), ref[1]), f"queued search {i}"
    # half the batch: the coarse kernel then runs its 64-row tile
    say("C5: search nq=64 nprobe=16 k=10")
    got = gpu_search(dw.index, q[:64], 16, 10)
    res = check_large(dw, q[:64], 16, 10, got, rows=[1, 33, 62])
    _check_assignment_sample(dw, nsample_lists=8, nvec=2000)
    _check_readback(dw, [w.nlist - 1])
    info = dw.index.info()
    assert info.n == w.n and info.index_bytes >= w.n * w.d * 2
    dw.index.close()
