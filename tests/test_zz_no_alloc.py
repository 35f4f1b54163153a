"""ivf_search_noalloc — the entry point for callers that cannot allocate device memory —
against ivf_search through the C ABI: same kernels, so every row must be bit-identical,
on two calls in a row (the second smaller, so stale contents of the shared static array
lie behind it), across indexes that share the array, and past its size limit."""
import numpy as np
import pytest

from paper_2504_15302_amd import ivf
from paper_2504_15302_amd import workloads as W
from tests.gpu_util import check_against_oracle, gpu_search, say, upload_host_index

pytestmark = pytest.mark.gpu


def _noalloc(idx, q, nprobe, k, stream=None, check_free=True):
    """One call through the C ABI; the device's free memory (hipMemGetInfo, which also sees
    the library's own allocations) must not move across it.  The first launch of a kernel in
    a process loads its code object, so the very first call is exempt."""
    import torch
    qd = torch.from_numpy(np.ascontiguousarray(q, dtype=np.float32)).cuda()
    out_i = torch.full((q.shape[0], k), -7, dtype=torch.int64, device="cuda")
    out_s = torch.full((q.shape[0], k), np.nan, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    idx.search_noalloc(qd, nprobe, k, out_i, out_s, stream=stream)
    torch.cuda.synchronize()
    if check_free:
        assert torch.cuda.mem_get_info()[0] == free_before
    return out_i.cpu().numpy(), out_s.cpu().numpy()


def test_noalloc_matches_ivf_search_on_two_calls_in_a_row_the_second_smaller():
    w = W.CONFIGS["C1"]
    h = W.build_host_index(w)
    idx = upload_host_index(h)
    q1 = W.queries(w, batch=11, nq=48)
    q2 = W.queries(w, batch=12, nq=5)
    say("no-alloc search: nq=48 nprobe=12 k=100, then nq=5 nprobe=3 k=7")
    got1 = _noalloc(idx, q1, 12, 100, check_free=False)
    info_scratch = idx.info().scratch_bytes
    assert info_scratch == 0                                   # nothing was allocated for it
    got2 = _noalloc(idx, q2, 3, 7)
    ref1 = gpu_search(idx, q1, 12, 100)
    ref2 = gpu_search(idx, q2, 3, 7)
    assert np.array_equal(got1[0], ref1[0]) and np.array_equal(got1[1], ref1[1])
    assert np.array_equal(got2[0], ref2[0]) and np.array_equal(got2[1], ref2[1])
    check_against_oracle(h.centroids, h.vectors, h.ids, h.offsets, q2, 3, 7, (got2[0], got2[1], ref2[2], ref2[3]), w.storage)
    # once more after the allocating entry point has run, and with host-resident lists read in place
    idx.set_device_budget(idx.info().index_bytes // 3)
    again = _noalloc(idx, q1, 12, 100)
    assert np.array_equal(again[0], ref1[0]) and np.array_equal(again[1], ref1[1])
    idx.close()


def test_noalloc_indexes_share_the_array_and_the_limit_is_an_error():
    import torch
    w = W.scaled(W.CONFIGS["C1"], n=40_000, nlist=96, name="C1-small")
    ha, hb = W.build_host_index(w), W.build_host_index(W.scaled(w, seed=w.seed + 77, storage="fp16"))
    ia, ib = upload_host_index(ha), upload_host_index(hb)
    qa, qb = W.queries(w, batch=1, nq=20), W.queries(w, batch=2, nq=9)
    ra, rb = gpu_search(ia, qa, 6, 10), gpu_search(ib, qb, 4, 25)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    da, db = torch.from_numpy(qa).cuda(), torch.from_numpy(qb).cuda()
    outs = []
    torch.cuda.synchronize()
    say("no-alloc searches of two indexes alternating on two streams")
    for rep in range(10):
        oa = (torch.empty((20, 10), dtype=torch.int64, device="cuda"), torch.empty((20, 10), dtype=torch.float32, device="cuda"))
        ob = (torch.empty((9, 25), dtype=torch.int64, device="cuda"), torch.empty((9, 25), dtype=torch.float32, device="cuda"))
        ia.search_noalloc(da, 6, 10, *oa, stream=sa)
        ib.search_noalloc(db, 4, 25, *ob, stream=sb)
        outs += [(ra, oa), (rb, ob)]
    torch.cuda.synchronize()
    for ref, (ids, sc) in outs:
        assert np.array_equal(ids.cpu().numpy(), ref[0]) and np.array_equal(sc.cpu().numpy(), ref[1])
    say("no-alloc search beyond the static array: nq=60000")
    big = torch.zeros((60000, w.d), dtype=torch.float32, device="cuda")
    oi = torch.empty((60000, 1), dtype=torch.int64, device="cuda")
    os_ = torch.empty((60000, 1), dtype=torch.float32, device="cuda")
    with pytest.raises(ivf.IvfError) as e:
        ia.search_noalloc(big, 96, 1, oi, os_)
    assert e.value.code == -5 and "static array" in str(e.value)
    # refused in the staged host-list mode, fine again afterwards
    ia.set_option("host_direct", 0)
    ia.set_device_budget(ia.info().index_bytes // 2)
    with pytest.raises(ivf.IvfError) as e:
        ia.search_noalloc(da, 6, 10, *outs[0][1])
    assert e.value.code == -1
    ia.set_option("host_direct", 1)
    ia.search_noalloc(da, 6, 10, *outs[0][1])
    torch.cuda.synchronize()
    assert np.array_equal(outs[0][1][0].cpu().numpy(), ra[0])
    ia.close()
    ib.close()
