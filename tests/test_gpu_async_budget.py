"""GPU tests of budget changes carried out in the background (the paper releases and loads
database partitions lazily, during the retrieval phase: Section 5 "Lazy dynamic transfer"):
searches issued at any point of a change give the same rows as before it, the change ends
in the placement the blocking call reaches, and memory is handed back."""
import threading

import numpy as np
import pytest

from paper_2504_15302_amd import ivf
from paper_2504_15302_amd import workloads as W
from tests.gpu_util import check_against_oracle, gpu_search, say, upload_host_index

pytestmark = pytest.mark.gpu

SEG = 64 << 20          # C1 is smaller than 16 segments of 64 MiB, so that is its segment size


@pytest.fixture(scope="module")
def c1():
    w = W.CONFIGS["C1"]
    h = W.build_host_index(w)
    say("C1: uploading 100k x 384 fp32 (asynchronous budget tests)")
    idx = upload_host_index(h)
    # small batches of copies, so that a change of this small index takes many steps
    idx.set_option("move_chunk_kb", 2048)
    idx.set_option("move_inflight_kb", 8192)
    return w, h, idx


def _resident_set(w, h, budget):
    lens = np.diff(h.offsets)
    nblk = (lens + 63) // 64
    bb = 64 * w.d * 4
    order = np.lexsort((np.arange(w.nlist), -lens))
    used, keep = 0, set()
    for l in order:
        b = int(nblk[l]) * bb
        if used + b > budget:
            break
        used += b
        keep.add(int(l))
    return keep, sum(int(nblk[l]) * bb for l in keep)


def _same(got, ref):
    return np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])


def test_searches_during_a_background_change_see_one_valid_place_per_list(c1):
    w, h, idx = c1
    q = W.queries(w, batch=11)
    ref = gpu_search(idx, q, w.nprobe, w.k)
    check_against_oracle(h.centroids, h.vectors, h.ids, h.offsets, q, w.nprobe, w.k, ref, w.storage)
    total = idx.info().index_bytes
    cur = set(range(w.nlist))
    try:
        for frac in (0.25, 1.0, 0.0, 0.6):
            budget = int(total * frac)
            want, res_b = _resident_set(w, h, budget)
            say(f"C1 background change to {frac:.2f} of the index: {len(want)} lists resident at the end")
            idx.set_device_budget_async(budget)
            steps, seen_partial, last_pending = 0, 0, None
            while True:
                pl, pb, busy = idx.budget_progress()
                if last_pending is not None:
                    assert pl <= last_pending            # lists only ever get nearer to their target
                last_pending = pl
                if not busy:
                    break
                got = gpu_search(idx, q, w.nprobe, w.k)
                assert _same(got, ref), f"rows changed {steps} searches into the change to {frac}"
                st = idx.last_search_stats()
                assert st.scan_bytes_resident + st.scan_bytes_streamed == st.scan_bytes
                r = idx.info().resident_lists
                seen_partial += 0 < abs(r - len(cur)) < abs(len(want) - len(cur))
                steps += 1
                assert steps < 5000
            say(f"  done after {steps} searches, {seen_partial} of them half-way")
            assert steps >= 3 and seen_partial >= 1      # the change really was spread over searches
            info = idx.info()
            assert info.resident_lists == len(want)
            assert info.device_list_bytes == res_b and info.host_list_bytes == total - res_b
            lens = np.diff(h.offsets)
            bb = 64 * w.d * 4
            nb = (lens + 63) // 64
            assert info.moved_d2h_bytes == sum(int(nb[l]) * bb for l in cur - want)
            assert info.moved_h2d_bytes == sum(int(nb[l]) * bb for l in want - cur)
            assert res_b <= info.device_pool_bytes <= res_b + 2 * SEG     # memory handed back
            assert total - res_b <= info.host_pool_bytes <= total - res_b + 2 * SEG
            got = gpu_search(idx, q, w.nprobe, w.k)
            assert _same(got, ref)
            for l in (0, 77, 255):
                vec, ids = idx.read_list(l, w.d, ivf.IVF_FP32)
                assert np.array_equal(vec, h.vectors[h.offsets[l]:h.offsets[l + 1]])
                assert np.array_equal(ids, h.ids[h.offsets[l]:h.offsets[l + 1]])
            cur = want
    finally:
        idx.set_device_budget(2**62)


def test_searches_queued_back_to_back_during_a_change(c1):
    """No host synchronisation between searches: the address table updates and the release
    of old places are ordered on the device alone."""
    import torch
    w, h, idx = c1
    qs = [torch.from_numpy(W.queries(w, batch=20 + i)).cuda() for i in range(3)]
    refs = []
    for qd in qs:
        ids, sc = idx.search(qd, w.nprobe, w.k)
        torch.cuda.synchronize()
        refs.append((ids.cpu().numpy(), sc.cpu().numpy()))
    total = idx.info().index_bytes
    try:
        for frac in (0.2, 1.0):
            say(f"C1 background change to {frac:.2f}, searches queued without synchronising")
            idx.set_device_budget_async(int(total * frac))
            rounds = 0
            while idx.budget_progress()[2]:
                outs = []
                for rep in range(4):
                    for i, qd in enumerate(qs):
                        outs.append((i, idx.search(qd, w.nprobe, w.k)))
                torch.cuda.synchronize()
                for i, (ids, sc) in outs:
                    assert np.array_equal(ids.cpu().numpy(), refs[i][0]) and np.array_equal(sc.cpu().numpy(), refs[i][1])
                rounds += 1
                assert rounds < 2000
            say(f"  done after {rounds} rounds of 12 searches")
            assert rounds >= 2
    finally:
        idx.set_device_budget(2**62)


def test_staged_copies_during_a_background_change(c1):
    w, h, idx = c1
    q = W.queries(w, batch=12)
    ref = gpu_search(idx, q, w.nprobe, w.k)
    total = idx.info().index_bytes
    try:
        idx.set_option("host_direct", 0)
        idx.set_option("stage_mb", 2)
        for frac in (0.3, 0.9, 0.0):
            say(f"C1 background change to {frac:.2f} with staged copies of host lists")
            idx.set_device_budget_async(int(total * frac))
            steps = 0
            while idx.budget_progress()[2]:
                got = gpu_search(idx, q, w.nprobe, w.k)
                assert _same(got, ref), f"rows changed {steps} searches into the change to {frac}"
                steps += 1
                assert steps < 5000
            assert steps >= 3
            assert _same(gpu_search(idx, q, w.nprobe, w.k), ref)
        with pytest.raises(ivf.IvfError):
            idx.set_device_budget_async(total)
            idx.set_option("host_direct", 1)          # not while a change is in progress
        idx.budget_wait()
    finally:
        idx.budget_wait()
        idx.set_option("host_direct", 1)
        idx.set_option("stage_mb", 64)
        idx.set_device_budget(2**62)


def test_a_new_target_or_a_blocking_call_half_way(c1):
    w, h, idx = c1
    q = W.queries(w, batch=13)
    ref = gpu_search(idx, q, w.nprobe, w.k)
    total = idx.info().index_bytes
    try:
        say("C1 background change to 0, new target 0.5 after three searches")
        idx.set_device_budget_async(0)
        for _ in range(3):
            assert _same(gpu_search(idx, q, w.nprobe, w.k), ref)
        assert 0 < idx.info().resident_lists < w.nlist
        idx.set_device_budget_async(int(total * 0.5))
        assert _same(gpu_search(idx, q, w.nprobe, w.k), ref)
        idx.budget_wait()
        pl, pb, busy = idx.budget_progress()
        assert (pl, pb, busy) == (0, 0, False)
        want, res_b = _resident_set(w, h, int(total * 0.5))
        info = idx.info()
        assert info.resident_lists == len(want) and info.device_list_bytes == res_b
        assert _same(gpu_search(idx, q, w.nprobe, w.k), ref)

        say("C1 background change to 0.1, blocking call to 0.8 half-way")
        idx.set_device_budget_async(int(total * 0.1))
        for _ in range(2):
            assert _same(gpu_search(idx, q, w.nprobe, w.k), ref)
        idx.set_device_budget(int(total * 0.8))
        assert not idx.budget_progress()[2]
        want, res_b = _resident_set(w, h, int(total * 0.8))
        info = idx.info()
        assert info.resident_lists == len(want) and info.device_list_bytes == res_b
        assert res_b <= info.device_pool_bytes <= res_b + 2 * SEG
        assert _same(gpu_search(idx, q, w.nprobe, w.k), ref)
        for l in range(0, w.nlist, 37):
            vec, ids = idx.read_list(l, w.d, ivf.IVF_FP32)
            assert np.array_equal(vec, h.vectors[h.offsets[l]:h.offsets[l + 1]])
    finally:
        idx.set_device_budget(2**62)


def test_evictions_and_loads_in_one_change_under_the_hot_policy():
    """Ranking by probe count swaps lists both ways in one change; fp16 storage, ragged
    and empty lists."""
    rng = np.random.default_rng(77)
    nlist, d, n = 96, 64, 30000
    cen = rng.standard_normal((nlist, d)).astype(np.float32)
    x = rng.standard_normal((n, d)).astype(np.float32)
    sc = x.astype(np.float64) @ cen.astype(np.float64).T
    sc[:, [5, 50]] = -np.inf                                  # two empty lists
    lab = np.argmax(sc, axis=1)
    o = np.argsort(lab, kind="stable")
    x, lab = x[o], lab[o]
    off = np.zeros(nlist + 1, dtype=np.int64)
    np.cumsum(np.bincount(lab, minlength=nlist), out=off[1:])
    ids = rng.permutation(3 * n)[:n].astype(np.int64)
    vec = np.ascontiguousarray(x.astype(np.float16))
    idx = ivf.Index()
    idx.set_option("segment_mb", 1)
    idx.upload(cen, vec, ids, off)
    idx.set_option("move_chunk_kb", 64)
    idx.set_option("move_inflight_kb", 256)
    q = rng.standard_normal((24, d)).astype(np.float32)
    nprobe, k = 6, 15
    ref = gpu_search(idx, q, nprobe, k)
    floor = float(np.linalg.norm(q, axis=1).max() * np.linalg.norm(vec.astype(np.float32), axis=1).max())
    check_against_oracle(cen, vec, ids, off, q, nprobe, k, ref, "fp16", abs_floor=floor)
    total = idx.info().index_bytes
    say("random fp16 index: length-ranked 40 % resident, then probe-ranked 40 % in the background")
    idx.set_device_budget(int(total * 0.4))
    assert _same(gpu_search(idx, q, nprobe, k), ref)
    streamed_by_length = idx.last_search_stats().scan_bytes_streamed
    idx.set_option("residency_policy", 1)
    idx.set_device_budget_async(int(total * 0.4))
    steps = 0
    while idx.budget_progress()[2]:
        assert _same(gpu_search(idx, q, nprobe, k), ref)
        steps += 1
        assert steps < 5000
    info = idx.info()
    assert info.moved_d2h_bytes > 0 and info.moved_h2d_bytes > 0     # lists went both ways
    assert _same(gpu_search(idx, q, nprobe, k), ref)
    # probed lists are now ranked first: less of the scan crosses PCIe than before
    assert idx.last_search_stats().scan_bytes_streamed < streamed_by_length
    for l in range(nlist):
        v, i = idx.read_list(l, d, ivf.IVF_FP16)
        assert np.array_equal(v, vec[off[l]:off[l + 1]]) and np.array_equal(i, ids[off[l]:off[l + 1]])
    say(f"  {steps} searches during the change; seeded random budgets next")
    for step in range(6):
        b = int(total * float(rng.uniform(0, 1.1)))
        idx.set_device_budget_async(b)
        for _ in range(int(rng.integers(0, 4))):
            assert _same(gpu_search(idx, q, nprobe, k), ref)
    idx.budget_wait()
    assert _same(gpu_search(idx, q, nprobe, k), ref)
    idx.close()


def test_the_worker_changes_the_budget_while_it_serves_requests(c1):
    w, h, idx = c1
    q = W.queries(w, batch=14, nq=96)
    ref = gpu_search(idx, q, w.nprobe, w.k)
    total = idx.info().index_bytes
    want, _ = _resident_set(w, h, int(total * 0.3))
    wk = ivf.Worker(idx, w.nprobe, w.k, 16)
    try:
        say("worker: 96 requests from three threads, budget change to 0.30 asked for meanwhile")
        results = {}

        def client(lo, hi):
            tickets = [(i, wk.submit(q[i])) for i in range(lo, hi)]
            for i, t in tickets:
                results[i] = wk.wait(t)

        th = [threading.Thread(target=client, args=(a, a + 32)) for a in (0, 32, 64)]
        th[0].start()
        wk.set_device_budget(int(total * 0.3))
        for t in th[1:]:
            t.start()
        for t in th:
            t.join(timeout=120)
            assert not t.is_alive()
        for i in range(96):
            assert np.array_equal(results[i][0], ref[0][i]) and np.array_equal(results[i][1], ref[1][i])
        import time
        t0 = time.time()
        while wk.stats().budget_busy and time.time() - t0 < 60:    # an idle worker finishes the change
            time.sleep(0.01)
        st = wk.stats()
        assert st.budget_busy == 0 and st.budget_error == 0 and st.budget_changes == 1
        assert st.resident_lists == len(want) and st.budget_pending_lists == 0
        # more requests after the change
        tickets = [wk.submit(q[i]) for i in range(8)]
        for i, t in enumerate(tickets):
            r = wk.wait(t)
            assert np.array_equal(r[0], ref[0][i]) and np.array_equal(r[1], ref[1][i])
        # a change asked for just before the stop is seen through
        wk.set_device_budget(2**62)
    finally:
        wk.stop()
    assert idx.info().resident_lists == w.nlist
    assert _same(gpu_search(idx, q, w.nprobe, w.k), ref)
