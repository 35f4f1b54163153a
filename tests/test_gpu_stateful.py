"""A seeded random walk over the library's state on the GPU: searches of several shapes
interleaved with blocking and background budget changes, policy and mode switches, scan
options, timing on and off, and a re-upload.  Whatever the state, a search returns the rows
it returned at the start (which are checked against the CPU oracle), every list reads back
intact, and the bookkeeping reported by ivf_get_info stays consistent."""
import numpy as np
import pytest

from paper_2504_15302_amd import ivf
from tests.gpu_util import check_against_oracle, gpu_search, say

pytestmark = pytest.mark.gpu


def _index(seed, storage):
    rng = np.random.default_rng(seed)
    nlist, d, n = 40, 48, 24000
    cen = rng.standard_normal((nlist, d)).astype(np.float32)
    x = rng.standard_normal((n, d)).astype(np.float32)
    sc = x.astype(np.float64) @ cen.astype(np.float64).T
    sc[:, [3, 17]] = -np.inf                                  # two empty lists
    sc[:, 5] += 1.5                                           # one list much longer than the rest
    lab = np.argmax(sc, axis=1)
    o = np.argsort(lab, kind="stable")
    x, lab = x[o], lab[o]
    off = np.zeros(nlist + 1, dtype=np.int64)
    np.cumsum(np.bincount(lab, minlength=nlist), out=off[1:])
    ids = rng.permutation(4 * n)[:n].astype(np.int64)
    if storage == "int8":
        from paper_2504_15302_amd import workloads as W
        vec = W.quantize_int8_host(x)
    else:
        vec = np.ascontiguousarray(x.astype(np.float16 if storage == "fp16" else np.float32))
    return cen, vec, ids, off


@pytest.mark.parametrize("seed,storage", [(1, "fp16"), (2, "fp32"), (3, "int8"), (4, "fp16"), (5, "int8")])
def test_random_walk_over_the_library_state(seed, storage):
    cen, vec, ids, off = _index(100 + seed, storage)
    rng = np.random.default_rng(seed)
    d = cen.shape[1]
    dt = {"fp32": ivf.IVF_FP32, "fp16": ivf.IVF_FP16, "int8": ivf.IVF_INT8}[storage]
    idx = ivf.Index()
    idx.set_option("segment_mb", 1)                           # several segments: compaction has work
    idx.upload(cen, vec, ids, off)
    idx.set_option("move_chunk_kb", 64)
    idx.set_option("move_inflight_kb", 256)
    total = idx.info().index_bytes
    shapes = [(5, 4, 10), (37, 7, 3), (1, 40, 100), (70, 2, 129)]        # nq, nprobe, k
    queries = [rng.standard_normal((nq, d)).astype(np.float32) for nq, _, _ in shapes]
    refs = []
    for q, (nq, nprobe, k) in zip(queries, shapes):
        got = gpu_search(idx, q, nprobe, k)
        if storage == "int8":
            from paper_2504_15302_amd import workloads as W
            codes, scales = W.split_int8_records(vec)
            floor = float(np.linalg.norm(q, axis=1).max() * (np.linalg.norm(codes.astype(np.float32), axis=1) * scales).max())
        else:
            floor = float(np.linalg.norm(q, axis=1).max() * np.linalg.norm(vec.astype(np.float32), axis=1).max())
        check_against_oracle(cen, vec, ids, off, q, nprobe, k, got, storage, abs_floor=floor)
        refs.append(got)
    direct, log = 1, []

    import torch
    idx.set_option("queue_min_mb", 0)                         # queued searches overlap however small they are
    own = torch.cuda.Stream()
    q_dev = [torch.from_numpy(q).cuda() for q in queries]
    q_pin = [torch.from_numpy(q).pin_memory() for q in queries]

    def search(i):
        """One of the entry points, by lot: plain; two queued searches back to back on a stream of
        the test's; queued with queries and results in pinned host memory; no allocation (refused
        during a budget change and in the staged mode: then plain)."""
        nq, nprobe, k = shapes[i]
        mode = int(rng.integers(0, 4))
        log[-1] += "/" + ("plain", "queued", "pinned", "noalloc")[mode]
        if mode == 1:
            outs = [idx.search_queued(q_dev[i], nprobe, k, stream=own) for _ in range(2)]
            own.synchronize()
            got = [(a.cpu().numpy(), b.cpu().numpy()) for a, b in outs]
        elif mode == 2:
            hi = torch.full((nq, k), -7, dtype=torch.int64).pin_memory()
            hs = torch.full((nq, k), np.nan, dtype=torch.float32).pin_memory()
            idx.search_queued(q_pin[i], nprobe, k, hi, hs, stream=own)
            own.synchronize()
            got = [(hi.numpy(), hs.numpy())]
        else:
            got = None
            if mode == 3:
                di = torch.empty((nq, k), dtype=torch.int64, device="cuda")
                ds = torch.empty((nq, k), dtype=torch.float32, device="cuda")
                try:
                    idx.search_noalloc(q_dev[i], nprobe, k, di, ds, stream=own)
                    own.synchronize()
                    got = [(di.cpu().numpy(), ds.cpu().numpy())]
                except ivf.IvfError as e:
                    assert "budget change" in str(e) or "staged" in str(e), str(e)
            if got is None:
                got = [gpu_search(idx, queries[i], nprobe, k)]
        for g in got:
            assert np.array_equal(g[0], refs[i][0]) and np.array_equal(g[1], refs[i][1]), \
                f"shape {shapes[i]} changed after: {log[-12:]}"

    for step in range(300):
        op = int(rng.integers(0, 100))
        if op < 45:
            i = int(rng.integers(0, len(shapes)))
            log.append(f"search{i}")
            search(i)
        elif op < 60:
            frac = float(rng.choice([0.0, 0.1, 0.35, 0.7, 1.0, 1.3]))
            log.append(f"budget {frac}")
            idx.set_device_budget(int(total * frac))
        elif op < 78:
            frac = float(rng.choice([0.0, 0.2, 0.5, 0.9, 1.2]))
            log.append(f"budget_async {frac}")
            idx.set_device_budget_async(int(total * frac))
        elif op < 82:
            log.append("wait")
            idx.budget_wait()
        elif op < 87:
            pol = int(rng.integers(0, 2))
            log.append(f"policy {pol}")
            idx.set_option("residency_policy", pol)
        elif op < 91:
            if not idx.budget_progress()[2]:
                direct ^= 1
                log.append(f"host_direct {direct}")
                idx.set_option("host_direct", direct)
                idx.set_option("stage_mb", int(rng.choice([1, 4, 64])))
        elif op < 95:
            name, values = [("scan_unroll", (8, 16)), ("scan_waves", (1, 2, 4, 8)), ("nside", (1, 2, 3)),
                            ("scan_prune", (0, 1, 2)), ("sel_threads", (0, 256, 1024)),
                            ("regroup_fused", (0, 1))][int(rng.integers(0, 6))]
            v = int(rng.choice(values))
            log.append(f"{name} {v}")
            idx.set_option(name, v)
        elif op < 98:
            on = bool(rng.integers(0, 2))
            log.append(f"timing {on}")
            idx.set_timing(on)
        else:
            log.append("re-upload")
            idx.upload(cen, vec, ids, off)
            total = idx.info().index_bytes
        if step % 10 == 9:
            info = idx.info()
            assert info.device_list_bytes + info.host_list_bytes == total
            assert info.device_list_bytes <= info.device_pool_bytes and info.host_list_bytes <= info.host_pool_bytes
            assert 0 <= info.resident_lists <= cen.shape[0]
            l = int(rng.integers(0, cen.shape[0]))
            v, i = idx.read_list(l, d, dt)
            assert np.array_equal(v, vec[off[l]:off[l + 1]]) and np.array_equal(i, ids[off[l]:off[l + 1]]), \
                f"list {l} damaged after: {log[-12:]}"
    idx.budget_wait()
    for i in range(len(shapes)):
        log.append(f"search{i}")
        search(i)
    say(f"random walk seed {seed} ({storage}): {len(log)} operations, last: {log[-6:]}")
    idx.close()
