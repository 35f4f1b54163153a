"""Retrieval worker (request queue -> batches -> context queue, paper Section 4.1):
every request is answered exactly once, with the result a direct ivf_search gives."""
import threading

import numpy as np
import pytest

from paper_2504_15302_amd import ivf
from paper_2504_15302_amd import workloads as W
from tests.gpu_util import gpu_search, say, upload_host_index

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def small():
    w = W.scaled(W.CONFIGS["C1"], n=40_000, nlist=128)
    h = W.build_host_index(w)
    return w, h, upload_host_index(h)


def test_worker_answers_every_request_once_with_the_direct_result(small):
    w, h, idx = small
    nthreads, per = 4, 80
    q = W.queries(w, batch=11, nq=nthreads * per)
    say("direct search of all worker queries")
    ref_ids, ref_scores, _, _ = gpu_search(idx, q, w.nprobe, w.k)
    worker = ivf.Worker(idx, w.nprobe, w.k, max_batch=64)
    tickets = [None] * len(q)
    results = [None] * len(q)

    def client(t):
        rng = np.random.default_rng(t)
        mine = list(range(t * per, (t + 1) * per))
        for i in mine:
            tickets[i] = worker.submit(q[i])
            if rng.random() < 0.2:                       # sometimes take a result right away
                results[i] = worker.wait(tickets[i])
        for i in mine:
            if results[i] is None:
                results[i] = worker.wait(tickets[i], timeout_ms=20000)

    say(f"{nthreads} client threads x {per} requests through the worker")
    th = [threading.Thread(target=client, args=(t,)) for t in range(nthreads)]
    for t in th:
        t.start()
    for t in th:
        t.join(60)
    assert all(not t.is_alive() for t in th)
    assert len(set(tickets)) == len(q)
    for i in range(len(q)):
        assert results[i] is not None, f"request {i} got no answer"
        assert np.array_equal(results[i][0], ref_ids[i]) and np.array_equal(results[i][1], ref_scores[i])
    st = worker.stats()
    assert st.requests_submitted == len(q) and st.requests_done == len(q)
    assert st.queued == 0 and st.results_waiting == 0 and 1 <= st.batches <= len(q)
    with pytest.raises(ivf.IvfError):                    # a ticket can be taken only once
        worker.wait(tickets[0], timeout_ms=10)
    with pytest.raises(ivf.IvfError):                    # unknown ticket
        worker.wait(10 ** 9, timeout_ms=10)

    # a backlog: many requests at once are served in batches, and the stop call drains the queue
    say("backlog of 300 requests")
    q2 = W.queries(w, batch=12, nq=300)
    t2 = [worker.submit(x) for x in q2]
    out2 = [worker.wait(t, timeout_ms=20000) for t in t2]
    st = worker.stats()
    assert st.requests_done == len(q) + 300 and st.largest_batch > 1 and st.largest_batch <= 64
    worker.stop()
    r_ids, r_scores, _, _ = gpu_search(idx, q2, w.nprobe, w.k)
    for i in range(300):
        assert np.array_equal(out2[i][0], r_ids[i]) and np.array_equal(out2[i][1], r_scores[i])
    say(f"worker ok: {st.batches} batches, largest {st.largest_batch}, fit c = {st.fit_c:.2f}")


def test_worker_rejects_bad_arguments(small):
    w, h, idx = small
    with pytest.raises(ivf.IvfError):
        ivf.Worker(idx, 0, 5, 8)
    with pytest.raises(ivf.IvfError):
        ivf.Worker(idx, 4, 5, 0)
    with pytest.raises(ivf.IvfError):
        ivf.Worker(ivf.Index(), 4, 5, 8)                 # no data uploaded
