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
    dt = {"fp32": ivf.IVF_FP32, "fp16": ivf.IVF_FP16, "int8": ivf.IVF_INT8}[w.storage]
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
