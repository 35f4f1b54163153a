"""Searches queued back to back: ivf_search_queued overlaps the stages of neighbouring
searches on the library's own streams and three sets of scratch memory, and consecutive
searches of one index may be issued on different streams.  Rows must be bit-identical to
those of ivf_search issued one by one (results never depend on batching or scheduling:
paper Section 6.1 "Key Metrics")."""
import numpy as np
import pytest

from paper_2504_15302_amd import ivf
from paper_2504_15302_amd import workloads as W
from tests.gpu_util import check_against_oracle, gpu_search, say, upload_host_index

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def c1():
    w = W.CONFIGS["C1"]
    h = W.build_host_index(w)
    say("C1: uploading 100k x 384 fp32")
    idx = upload_host_index(h)
    idx.set_option("queue_min_mb", 0)          # searches this small would otherwise stay on one stream
    yield w, h, idx
    idx.close()


def _refs(idx, w, nb, nq=None, nprobe=None, k=None):
    import torch
    qs = [W.queries(w, batch=20 + b, nq=nq or w.nq) for b in range(nb)]
    refs = [gpu_search(idx, q, nprobe or w.nprobe, k or w.k) for q in qs]
    return qs, [torch.from_numpy(q).cuda() for q in qs], refs


def test_queued_searches_equal_searches_issued_one_by_one(c1):
    import torch
    w, h, idx = c1
    qs, qd, refs = _refs(idx, w, 5)
    check_against_oracle(h.centroids, h.vectors, h.ids, h.offsets, qs[0], w.nprobe, w.k, refs[0], w.storage)
    torch.cuda.synchronize()
    say("C1: 40 queued searches, no host synchronisation in between")
    outs = []
    for i in range(40):
        outs.append(idx.search_queued(qd[i % 5], w.nprobe, w.k))
    torch.cuda.synchronize()
    for i, (ids, sc) in enumerate(outs):
        assert np.array_equal(ids.cpu().numpy(), refs[i % 5][0]), f"search {i}"
        assert np.array_equal(sc.cpu().numpy(), refs[i % 5][1]), f"search {i}"
    # introspection refers to the last search
    st = idx.last_search_stats()
    assert st.pairs == w.nq * w.nprobe
    assert np.array_equal(idx.last_probes(w.nq, w.nprobe).cpu().numpy(), refs[39 % 5][2])


def test_queued_searches_into_one_output_buffer_with_copies_between(c1):
    """The caller reuses out_ids / out_scores and copies them away on its stream between two
    searches: the next selection's writes must wait for that copy."""
    import torch
    w, h, idx = c1
    qs, qd, refs = _refs(idx, w, 4)
    out_i = torch.empty((w.nq, w.k), dtype=torch.int64, device="cuda")
    out_s = torch.empty((w.nq, w.k), dtype=torch.float32, device="cuda")
    st = torch.cuda.Stream()
    keep_i = [torch.empty((w.nq, w.k), dtype=torch.int64).pin_memory() for _ in range(24)]
    keep_s = [torch.empty((w.nq, w.k), dtype=torch.float32).pin_memory() for _ in range(24)]
    torch.cuda.synchronize()
    say("C1: 24 queued searches into the same output buffers, copied to the host in between")
    with torch.cuda.stream(st):
        for i in range(24):
            idx.search_queued(qd[i % 4], w.nprobe, w.k, out_i, out_s, stream=st)
            keep_i[i].copy_(out_i, non_blocking=True)
            keep_s[i].copy_(out_s, non_blocking=True)
    st.synchronize()
    for i in range(24):
        assert np.array_equal(keep_i[i].numpy(), refs[i % 4][0]) and np.array_equal(keep_s[i].numpy(), refs[i % 4][1]), f"search {i}"


def test_queries_ready_event_orders_the_read_of_the_queries(c1):
    """The queries arrive by a copy on another stream; the event recorded behind the copy is
    what the search waits for (stream order on `stream` does not cover them)."""
    import torch
    w, h, idx = c1
    qs, qd, refs = _refs(idx, w, 3)
    copy_stream, st = torch.cuda.Stream(), torch.cuda.Stream()
    pinned = [torch.from_numpy(q).pin_memory() for q in qs]
    bufs = [torch.zeros((w.nq, w.d), dtype=torch.float32, device="cuda") for _ in range(6)]
    torch.cuda.synchronize()
    say("C1: queued searches behind host-to-device copies of their queries")
    outs = []
    for i in range(6):
        ev = torch.cuda.Event()
        with torch.cuda.stream(copy_stream):
            bufs[i].copy_(pinned[i % 3], non_blocking=True)
            ev.record(copy_stream)
        outs.append(idx.search_queued(bufs[i], w.nprobe, w.k, stream=st, queries_ready=ev))
    torch.cuda.synchronize()
    for i, (ids, sc) in enumerate(outs):
        assert np.array_equal(ids.cpu().numpy(), refs[i % 3][0]) and np.array_equal(sc.cpu().numpy(), refs[i % 3][1]), f"search {i}"


def test_consecutive_searches_of_one_index_on_different_streams(c1):
    """ivf_search on alternating streams, queued and plain searches mixed, different shapes,
    never a host synchronisation: the library orders them on the device."""
    import torch
    w, h, idx = c1
    qs, qd, refs = _refs(idx, w, 3)
    qs2, qd2, refs2 = _refs(idx, w, 2, nq=40, nprobe=5, k=17)
    streams = [torch.cuda.Stream() for _ in range(3)]
    torch.cuda.synchronize()
    say("C1: plain searches on three alternating streams")
    outs = []
    for i in range(18):
        outs.append((refs[i % 3], idx.search(qd[i % 3], w.nprobe, w.k, stream=streams[i % 3])))
    torch.cuda.synchronize()
    for i, (ref, (ids, sc)) in enumerate(outs):
        assert np.array_equal(ids.cpu().numpy(), ref[0]) and np.array_equal(sc.cpu().numpy(), ref[1]), f"search {i}"
    say("C1: plain and queued searches mixed, streams and shapes alternating")
    rng = np.random.default_rng(3)
    outs = []
    for i in range(60):
        big = bool(rng.integers(2))
        queued = bool(rng.integers(2))
        s = streams[int(rng.integers(3))]
        j = int(rng.integers(2 if big else 3))
        q, ref, np_, k = (qd2[j], refs2[j], 5, 17) if big else (qd[j], refs[j], w.nprobe, w.k)
        fn = idx.search_queued if queued else idx.search
        outs.append((ref, fn(q, np_, k, stream=s)))
    torch.cuda.synchronize()
    for i, (ref, (ids, sc)) in enumerate(outs):
        assert np.array_equal(ids.cpu().numpy(), ref[0]) and np.array_equal(sc.cpu().numpy(), ref[1]), f"search {i}"


def test_queued_searches_through_budget_changes_and_placements(c1):
    """With host-resident lists, during a background budget change and in the staged mode
    queued searches run on one stream; rows never change."""
    import torch
    w, h, idx = c1
    qs, qd, refs = _refs(idx, w, 3)
    total = idx.info().index_bytes
    try:
        say("C1: queued searches with 30 % of the index in HBM")
        idx.set_device_budget(int(total * 0.3))
        outs = [idx.search_queued(qd[i % 3], w.nprobe, w.k) for i in range(12)]
        torch.cuda.synchronize()
        for i, (ids, sc) in enumerate(outs):
            assert np.array_equal(ids.cpu().numpy(), refs[i % 3][0]) and np.array_equal(sc.cpu().numpy(), refs[i % 3][1])
        say("C1: queued searches while the budget grows back in the background")
        idx.set_option("move_chunk_kb", 4096)
        idx.set_device_budget_async(2**62)
        outs, n = [], 0
        while idx.budget_progress()[2] and n < 400:
            outs.append((n % 3, idx.search_queued(qd[n % 3], w.nprobe, w.k)))
            n += 1
        idx.budget_wait()
        outs += [(i % 3, idx.search_queued(qd[i % 3], w.nprobe, w.k)) for i in range(6)]
        torch.cuda.synchronize()
        for j, (ids, sc) in outs:
            assert np.array_equal(ids.cpu().numpy(), refs[j][0]) and np.array_equal(sc.cpu().numpy(), refs[j][1])
        say("C1: queued searches in the staged host-list mode")
        idx.set_option("host_direct", 0)
        idx.set_device_budget(int(total * 0.5))
        outs = [idx.search_queued(qd[i % 3], w.nprobe, w.k) for i in range(6)]
        torch.cuda.synchronize()
        for i, (ids, sc) in enumerate(outs):
            assert np.array_equal(ids.cpu().numpy(), refs[i % 3][0]) and np.array_equal(sc.cpu().numpy(), refs[i % 3][1])
    finally:
        idx.set_option("host_direct", 1)
        idx.set_option("move_chunk_kb", 65536)
        idx.set_device_budget(2**62)


def test_queued_searches_at_a_larger_shape_with_pruning():
    """Enough blocks for the scan's store pruning (running per-query bounds live in the
    scratch set) and the unfused regrouping; k = 100 keeps two blocks per bound."""
    import torch
    w = W.scaled(W.CONFIGS["C2"], n=400_000, nlist=2048, name="C2-small")
    h = W.build_host_index(w)
    idx = upload_host_index(h)
    idx.set_option("scan_prune", 2)
    qs = [W.queries(w, batch=b) for b in range(3)]
    qd = [torch.from_numpy(q).cuda() for q in qs]
    refs = [gpu_search(idx, q, w.nprobe, 100) for q in qs]
    check_against_oracle(h.centroids, h.vectors, h.ids, h.offsets, qs[1], w.nprobe, 100, refs[1], w.storage)
    idx.set_timing(2)
    say("C2-small: 30 queued searches, k=100, pruning on, scan timed")
    outs = [idx.search_queued(qd[i % 3], w.nprobe, 100) for i in range(30)]
    torch.cuda.synchronize()
    for i, (ids, sc) in enumerate(outs):
        assert np.array_equal(ids.cpu().numpy(), refs[i % 3][0]) and np.array_equal(sc.cpu().numpy(), refs[i % 3][1]), f"search {i}"
    ms = idx.stage_ms(0)
    assert ms["scan"] > 0 and ms["coarse"] == 0
    idx.set_timing(0)
    idx.close()


def test_first_queued_searches_on_a_busy_stream():
    """The library picks its three streams by trial at the first queued search that finds the
    caller's stream idle; searches before that (here: ten on a stream that still has work)
    run on streams taken as they come, and after the eighth it stops waiting for an idle
    moment.  Rows are the same throughout, and the same again once the stream is idle."""
    import torch
    w = W.CONFIGS["C1"]
    h = W.build_host_index(w)
    say("C1: fresh index, first queued searches behind work on the caller's stream")
    idx = upload_host_index(h)
    try:
        idx.set_option("queue_min_mb", 0)
        qs, qd, refs = _refs(idx, w, 3)
        st = torch.cuda.Stream()
        a = torch.randn((4096, 4096), device="cuda")
        torch.cuda.synchronize()
        outs = []
        with torch.cuda.stream(st):
            for i in range(10):
                for _ in range(4):
                    a @ a                              # a few milliseconds ahead of every search
                outs.append(idx.search_queued(qd[i % 3], w.nprobe, w.k, stream=st))
        st.synchronize()
        for i in range(6):                             # idle now
            outs.append(idx.search_queued(qd[(10 + i) % 3], w.nprobe, w.k, stream=st))
        st.synchronize()
        for i, (ids, sc) in enumerate(outs):
            assert np.array_equal(ids.cpu().numpy(), refs[i % 3][0]), f"search {i}"
            assert np.array_equal(sc.cpu().numpy(), refs[i % 3][1]), f"search {i}"
    finally:
        idx.close()


def test_queries_and_results_in_pinned_host_memory(c1):
    """Queries handed over in pinned host memory are copied to the device by the search
    itself (on the stream of its first kernel), results may land in pinned host memory
    directly: same rows as with device buffers, for plain, queued and no-allocation
    searches; pageable host memory is refused."""
    import torch
    w, h, idx = c1
    qs, qd, refs = _refs(idx, w, 3)
    qp = [torch.from_numpy(q).pin_memory() for q in qs]
    st = torch.cuda.Stream()
    torch.cuda.synchronize()
    say("C1: pinned queries -> plain, queued (pinned results), no-allocation searches")
    for b in range(3):
        ids, sc = idx.search(qp[b], w.nprobe, w.k, stream=st)
        st.synchronize()
        assert np.array_equal(ids.cpu().numpy(), refs[b][0]) and np.array_equal(sc.cpu().numpy(), refs[b][1])
    outs = []
    for i in range(12):
        hi = torch.full((w.nq, w.k), -7, dtype=torch.int64).pin_memory()
        hs = torch.full((w.nq, w.k), np.nan, dtype=torch.float32).pin_memory()
        idx.search_queued(qp[i % 3], w.nprobe, w.k, hi, hs, stream=st)
        outs.append((hi, hs))
    st.synchronize()
    for i, (hi, hs) in enumerate(outs):
        assert np.array_equal(hi.numpy(), refs[i % 3][0]) and np.array_equal(hs.numpy(), refs[i % 3][1]), f"search {i}"
    di = torch.empty((w.nq, w.k), dtype=torch.int64, device="cuda")
    ds = torch.empty((w.nq, w.k), dtype=torch.float32, device="cuda")
    idx.search_noalloc(qp[1], w.nprobe, w.k, di, ds, stream=st)
    st.synchronize()
    assert np.array_equal(di.cpu().numpy(), refs[1][0]) and np.array_equal(ds.cpu().numpy(), refs[1][1])
    pageable = np.ascontiguousarray(qs[0])
    rc = idx._lib.ivf_search(idx._h, pageable.ctypes.data, w.nq, w.nprobe, w.k, di.data_ptr(), ds.data_ptr(), None)
    assert rc == -1 and b"pinned" in idx._lib.ivf_last_error()      # IVF_ERR_INVALID
