"""Generates a synthetic workload on the GPU and hands it to the library in pieces
(ivf_index_upload_begin / _lists / _end), so that an index of any size is never held
twice.  Used by the benchmark and by the full-size GPU tests."""
from __future__ import annotations

import time
from dataclasses import dataclass

import numpy as np

from . import ivf
from . import workloads as W


@dataclass
class LoadedWorkload:
    w: W.Workload
    index: ivf.Index
    centroids: np.ndarray     # host [nlist, d] float32
    offsets: np.ndarray       # host [nlist+1] int64
    centroids_dev: "object"   # torch tensor
    ids_dev: "object"         # torch tensor [n] int64, list-major
    seconds: float


def load_workload(w: W.Workload, groups_per_chunk: int = 16, log=None) -> LoadedWorkload:
    import torch
    t0 = time.time()
    cen = W.centroids(w)
    off = W.list_offsets(w)
    cen_dev = torch.from_numpy(cen).cuda()
    ids_dev = W.user_ids_device(w)
    index = ivf.Index()
    dt = {"fp32": ivf.IVF_FP32, "fp16": ivf.IVF_FP16, "int8": ivf.IVF_INT8, "pq8": ivf.IVF_PQ8}[w.storage]
    if w.storage == "pq8":
        index.set_pq_codebooks(W.pq_codebooks(w))
    index.upload_begin(cen, w.n, dt, off)
    last = t0
    for l0, l1, vec in W.iter_device_chunks(w, cen_dev, off, groups_per_chunk):
        r0, r1 = int(off[l0]), int(off[l1])
        index.upload_lists(l0, l1, vec, ids_dev[r0:r1].contiguous())
        del vec
        if log and time.time() - last > 20:
            log(f"{w.name}: uploaded lists [0,{l1}) of {w.nlist}")
            last = time.time()
    index.upload_end()
    torch.cuda.synchronize()
    return LoadedWorkload(w, index, cen, off, cen_dev, ids_dev, time.time() - t0)


def host_lists(lw: LoadedWorkload, lists):
    """Row-major host copy of the given lists, regenerated from the seeded recipe (not read
    back from the library): a compact sub-index (vectors, ids, offsets, global -> compact
    list number).  This is what the CPU oracle is fed with at the large configurations."""
    w, off = lw.w, lw.offsets
    lists = sorted(set(int(l) for l in lists))
    by_group = {}
    for l in lists:
        by_group.setdefault(l // W.GROUP, []).append(l)
    parts, idp, lens = {}, {}, {}
    for g, ls in by_group.items():
        gv = W.group_vectors_device(w, lw.centroids_dev, off, g, g + 1)
        base = int(off[g * W.GROUP])
        for l in ls:
            a, b = int(off[l]) - base, int(off[l + 1]) - base
            parts[l] = gv[a:b].cpu().numpy()
            idp[l] = lw.ids_dev[int(off[l]):int(off[l + 1])].cpu().numpy()
            lens[l] = b - a
        del gv
    coff = np.zeros(len(lists) + 1, dtype=np.int64)
    np.cumsum([lens[l] for l in lists], out=coff[1:])
    cols = w.d + 4 if w.storage == "int8" else w.pq_m if w.storage == "pq8" else w.d
    dt = {"fp32": np.float32, "fp16": np.float16, "int8": np.uint8, "pq8": np.uint8}[w.storage]
    vec = np.concatenate([parts[l] for l in lists], axis=0) if lists else np.empty((0, cols), dtype=dt)
    ids = np.concatenate([idp[l] for l in lists]) if lists else np.empty(0, np.int64)
    cmap = {l: i for i, l in enumerate(lists)}
    return vec, ids, coff, cmap
