"""Helpers of the GPU parity tests: run the HIP path through the C ABI binding and
compare it with the CPU oracle under the benchmark's correctness bar."""
from __future__ import annotations

import sys

import numpy as np

from oracle import check as CK
from oracle import ivf_oracle as O
from paper_2504_15302_amd import ivf
from paper_2504_15302_amd import workloads as W


def say(msg: str):
    """Progress line, flushed: names the case before each GPU step."""
    print(f"[gpu-test] {msg}", flush=True)
    sys.stdout.flush()


def gpu_search(index: ivf.Index, q: np.ndarray, nprobe: int, k: int):
    import torch
    qd = torch.from_numpy(np.ascontiguousarray(q, dtype=np.float32)).cuda()
    ids, scores = index.search(qd, nprobe, k)
    torch.cuda.synchronize()
    nprobe_eff = min(nprobe, index.info().nlist)
    probes = index.last_probes(q.shape[0], nprobe_eff)
    coarse = index.last_coarse(q.shape[0], index.info().nlist)
    torch.cuda.synchronize()
    return ids.cpu().numpy(), scores.cpu().numpy(), probes.cpu().numpy(), coarse.cpu().numpy()


def check_against_oracle(cen, vec, ids, off, q, nprobe, k, got, storage: str, extra_rows: int = 8,
                         abs_floor: float = 0.0, coarse_only_lists=None):
    """`got` = (ids, scores, probes, coarse) from gpu_search.  The index arrays are host
    NumPy arrays holding (at least) every probed list; list numbers are global."""
    g_ids, g_scores, g_probes, g_coarse = got
    nlist = cen.shape[0]
    nprobe = min(nprobe, nlist)
    o_coarse = O.coarse(q, cen)
    # stage 1: coarse scores, fp32 MFMA vs fp64: error bounded by ~d*eps*|q||c|
    scale = np.linalg.norm(q.astype(np.float64), axis=1)[:, None] * \
        np.linalg.norm(cen.astype(np.float64), axis=1)[None, :]
    err = np.abs(g_coarse.astype(np.float64) - o_coarse)
    assert (err <= 1e-5 * np.maximum(scale, 1e-30)).all(), \
        f"coarse scores off by up to {float((err / np.maximum(scale, 1e-30)).max()):.3g} of |q||c|"
    # stage 2: probe sets (order inside the set is checked when sets are equal)
    same = CK.check_probes(g_probes, o_coarse, nprobe)
    o_probes = O.probe_select(o_coarse, nprobe)
    if same:
        for r in range(q.shape[0]):
            if not np.array_equal(g_probes[r], o_probes[r]):
                # only near-tied neighbours may swap
                for a, b in zip(g_probes[r], o_probes[r]):
                    if a != b:
                        assert CK._near(float(o_coarse[r, a]), float(o_coarse[r, b]), CK.TIE_REL), \
                            f"q{r}: probe order differs beyond a near-tie"
        use = o_probes
    else:
        use = g_probes     # accepted near-tie at the probe boundary: oracle re-scans the GPU's set
    # stage 3: scan + selection
    o_ids, o_scores = O.scan_select(vec, ids, off, q, use, k + extra_rows)
    res = CK.check_topk(g_ids, g_scores, o_ids, o_scores, k, CK.SCORE_REL[storage], abs_floor=abs_floor)
    CK.check_ids_in_probed_lists(g_ids, use, ids, off)
    res["probe_sets_equal"] = bool(same)     # False: the oracle re-scanned the GPU's near-tied probe set
    return res


def upload_host_index(h: W.HostIndex) -> ivf.Index:
    idx = ivf.Index()
    idx.upload(h.centroids, h.vectors, h.ids, h.offsets)
    return idx


class DeviceWorkload:
    """A large synthetic index generated on the GPU and handed to the library piece by
    piece, plus what the oracle needs to re-derive any list on the host."""

    def __init__(self, w: W.Workload, groups_per_chunk: int = 16):
        from paper_2504_15302_amd.loader import load_workload
        lw = load_workload(w, groups_per_chunk, log=say)
        self.lw = lw
        self.w = w
        self.cen, self.off = lw.centroids, lw.offsets
        self.cen_dev, self.ids_dev, self.index = lw.centroids_dev, lw.ids_dev, lw.index
        say(f"{w.name}: generated and uploaded {w.n} x {w.d} {w.storage} in {lw.seconds:.1f}s")

    def host_lists(self, lists):
        """Row-major host copy of the given lists, regenerated from the seeded recipe
        (not read back from the library)."""
        from paper_2504_15302_amd.loader import host_lists
        return host_lists(self.lw, lists)


def check_large(dw: DeviceWorkload, q: np.ndarray, nprobe: int, k: int, got, rows=None, extra_rows: int = 8,
                row_chunk: int = 32):
    """Parity at full size: coarse scores and probe sets for every query (centroids are
    small), scan + selection for the query rows in `rows` (all if None), `row_chunk` rows
    at a time with only their probed lists brought to the host (regenerated from the
    seeded recipe), so that the host never holds more than a chunk's lists."""
    g_ids, g_scores, g_probes, g_coarse = got
    w = dw.w
    nprobe = min(nprobe, w.nlist)
    o_coarse = O.coarse(q, dw.cen)
    scale = np.linalg.norm(q.astype(np.float64), axis=1)[:, None] * \
        np.linalg.norm(dw.cen.astype(np.float64), axis=1)[None, :]
    err = np.abs(g_coarse.astype(np.float64) - o_coarse)
    assert (err <= 1e-5 * np.maximum(scale, 1e-30)).all(), "coarse scores off"
    same = CK.check_probes(g_probes, o_coarse, nprobe)
    use = O.probe_select(o_coarse, nprobe) if same else g_probes
    all_rows = list(range(q.shape[0])) if rows is None else list(rows)
    res = {"queries": 0, "tie_runs_reordered": 0, "probe_sets_equal": bool(same)}
    for c0 in range(0, len(all_rows), row_chunk):
        rows = all_rows[c0:c0 + row_chunk]
        vec, ids, coff, cmap = dw.host_lists(use[rows].ravel())
        cprobes = np.vectorize(cmap.get)(use[rows]).astype(np.int32)
        if w.storage == "pq8":       # the codes stand for decoded float32 vectors: the flat oracle over those
            from oracle import pq_oracle as PQ
            vec = PQ.decode(vec, W.pq_codebooks(w))
        o_ids, o_scores = O.scan_select(vec, ids, coff, q[rows], cprobes, k + extra_rows)
        r = CK.check_topk(g_ids[rows], g_scores[rows], o_ids, o_scores, k, CK.SCORE_REL[w.storage])
        CK.check_ids_in_probed_lists(g_ids[rows], cprobes, ids, coff)
        res["queries"] += r["queries"]
        res["tie_runs_reordered"] += r["tie_runs_reordered"]
        del vec, ids
        if len(all_rows) > row_chunk:
            say(f"{w.name}: rows {rows[0]}..{rows[-1]} match the oracle")
    # properties that hold for every row at any size
    assert np.all(g_scores[:, :-1] >= g_scores[:, 1:])
    for r in range(q.shape[0]):
        real = g_ids[r][g_ids[r] >= 0]
        assert len(np.unique(real)) == len(real)
    return res
