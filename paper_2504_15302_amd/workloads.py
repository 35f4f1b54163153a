"""Seeded synthetic workloads for the batched IVF retrieval path.

This module only *draws inputs*: Gaussian-mixture embeddings, their inverted-list
grouping, user ids and query batches.  It holds none of the retrieval arithmetic
(no similarity search, no probe selection, no k-selection) and is the one piece
shared by the HIP path's tests/bench and the CPU oracle's tests.

The paper's knowledge base (a TriviaQA-derived vector store of ~256 GB in 32
partitions, Section 6.1 "Dataset and Models") is not available and its embedding
model is not named, so these inputs stand in for it: same role (a chunk-embedding
store far larger than a query batch, batched queries, small k), shapes taken
from the benchmark configurations.

Recipe (per configuration, master seed S):
  * centroids  mu_c = g / |g|,  g ~ N(0, I_d)              (NumPy, stream 0)
  * list sizes (len_0..len_{nlist-1}) ~ Multinomial(n, uniform)  (NumPy, stream 1)
  * vectors of list c:  x = (mu_c + sigma * g) / |mu_c + sigma * g|, g ~ N(0, I_d),
    drawn per *group* of GROUP consecutive lists so that any group can be
    regenerated alone                                       (stream 2, group index)
  * queries: component c ~ Uniform{0..nlist-1}, same formula (stream 3, batch index)
  * user ids: a seeded permutation of 0..n-1 laid over the list-major order (stream 4)

A vector's list is the mixture component it was drawn from.  With these sigmas the
home centroid wins the arg-max inner product by more than ten standard deviations
of the cross-component score, so this equals "assigned to its argmax-IP centroid";
the tests check that equality with the oracle's assignment routine (all of C1,
samples of the larger configurations) instead of trusting it.

Two backends draw the normals: NumPy on the host (small configurations, usable
without a GPU) and torch on the device (large ones; the bytes never visit the
host).  They follow the same recipe but different random streams.
"""
from __future__ import annotations

import functools
from dataclasses import dataclass, replace
from typing import Iterator, Optional, Tuple

import numpy as np

GROUP = 64  # lists per generation group
_MASTER = 250415302

_STREAM_MEANS, _STREAM_SIZES, _STREAM_NOISE, _STREAM_QUERY, _STREAM_IDS, _STREAM_CODEBOOK = range(6)


@dataclass(frozen=True)
class Workload:
    name: str
    n: int
    d: int
    nlist: int
    sigma: float
    storage: str          # "fp32" | "fp16" | "int8" (records of d codes + fp32 scale) | "pq8" (pq_m codes)
    nq: int
    nprobe: int
    k: int
    seed: int
    resident_list_frac: Optional[float] = None  # None = everything HBM-resident
    pq_m: int = 0         # "pq8": number of subspaces (one byte of code each)
    uniform_lists: bool = False   # every list n / nlist vectors long (experiments on the effect of list length)

    @property
    def elem_bytes(self) -> int:
        return {"fp32": 4, "fp16": 2, "int8": 1, "pq8": 1}[self.storage]

    @property
    def row_bytes(self) -> int:
        """Bytes of one stored vector as uploaded."""
        if self.storage == "pq8":
            return self.pq_m
        return self.d * self.elem_bytes + (4 if self.storage == "int8" else 0)

    @property
    def ngroups(self) -> int:
        return (self.nlist + GROUP - 1) // GROUP


CONFIGS = {
    "C1": Workload("C1", 100_000, 384, 256, 0.05, "fp32", 16, 8, 10, _MASTER + 0),
    "C2": Workload("C2", 2_000_000, 768, 4096, 0.04, "fp32", 32, 32, 10, _MASTER + 1),
    "C3": Workload("C3", 20_000_000, 768, 16384, 0.04, "fp16", 64, 64, 20, _MASTER + 2),
    # same index and queries as C3 (first 8 of its 64), a quarter of the lists resident
    "C4": Workload("C4", 20_000_000, 768, 16384, 0.04, "fp16", 8, 64, 20, _MASTER + 2,
                   resident_list_frac=0.25),
    "C5": Workload("C5", 100_000_000, 768, 65536, 0.04, "fp16", 128, 128, 100, _MASTER + 4),
}
# The same indexes with compressed lists: every vector of the recipe, quantised to int8
# codes with one scale per vector (quantize_int8_*).  Same seeds, same queries.
for _name in ("C1", "C3", "C5"):
    CONFIGS[_name + "-int8"] = replace(CONFIGS[_name], name=_name + "-int8", storage="int8")


# ... and as product-quantisation codes: 8 dimensions per one-byte code (96 bytes per vector
# at d = 768, a sixteenth of the fp16 index), codebooks drawn from the same mixture.
for _name in ("C1", "C3", "C5"):
    CONFIGS[_name + "-pq"] = replace(CONFIGS[_name], name=_name + "-pq", storage="pq8",
                                     pq_m=CONFIGS[_name].d // 8)


def scaled(w: Workload, **kw) -> Workload:
    """A workload with some fields replaced (reduced sizes for quick tests)."""
    return replace(w, **kw)


def _rng(w: Workload, stream: int, index: int = 0) -> np.random.Generator:
    return np.random.default_rng([w.seed, stream, index])


def _torch_seed(w: Workload, stream: int, index: int) -> int:
    ss = np.random.SeedSequence([w.seed, stream, index])
    return int(ss.generate_state(1, dtype=np.uint64)[0] >> np.uint64(1))


def centroids(w: Workload) -> np.ndarray:
    """[nlist, d] float32 unit vectors: the mixture means, which are also the
    coarse-quantiser centroids."""
    g = _rng(w, _STREAM_MEANS).standard_normal((w.nlist, w.d))
    g /= np.linalg.norm(g, axis=1, keepdims=True)
    return np.ascontiguousarray(g.astype(np.float32))


def list_offsets(w: Workload) -> np.ndarray:
    """[nlist+1] int64 prefix sums of the multinomial list sizes."""
    if w.uniform_lists:
        assert w.n % w.nlist == 0
        sizes = np.full(w.nlist, w.n // w.nlist, dtype=np.int64)
    else:
        sizes = _rng(w, _STREAM_SIZES).multinomial(w.n, np.full(w.nlist, 1.0 / w.nlist))
    off = np.zeros(w.nlist + 1, dtype=np.int64)
    np.cumsum(sizes, out=off[1:])
    return off


def queries(w: Workload, batch: int = 0, nq: Optional[int] = None, components: Optional[int] = None,
            tight: bool = False) -> np.ndarray:
    """[nq, d] float32 unit query embeddings of batch number `batch`.  The first
    rows of a batch do not depend on nq, so C4's 8 queries are C3's first 8.
    With `components` = m the batch is skewed: its queries come from only m mixture
    components (drawn per batch), so about nq/m queries probe the same home list; with
    `tight` the queries of a component are near copies of one another (the component's
    first query plus a thousandth of the noise), so they probe the same lists throughout."""
    nq = w.nq if nq is None else nq
    cen = centroids(w)
    out = np.empty((nq, w.d), dtype=np.float32)
    hot = None
    if components is not None:
        hot = np.random.default_rng([w.seed, _STREAM_QUERY, batch, 1 << 20]).choice(w.nlist, size=components, replace=False)
    for i in range(nq):
        rng = np.random.default_rng([w.seed, _STREAM_QUERY, batch, i])
        comp = int(rng.integers(0, w.nlist))
        if hot is not None:
            comp = int(hot[comp % components])
        if hot is not None and tight:
            g0 = np.random.default_rng([w.seed, _STREAM_QUERY, batch, (1 << 21) + comp]).standard_normal(w.d).astype(np.float32)
            g = g0 + np.float32(1e-3) * rng.standard_normal(w.d).astype(np.float32)
            x = cen[comp] + np.float32(w.sigma) * g
            out[i] = x / np.linalg.norm(x)
            continue
        g = rng.standard_normal(w.d).astype(np.float32)
        x = cen[comp] + np.float32(w.sigma) * g
        out[i] = x / np.linalg.norm(x)
    return out


def quantize_int8_host(x: np.ndarray) -> np.ndarray:
    """Data preparation for int8 storage: [rows, d] float32 -> [rows, d+4] uint8 records
    of d signed codes followed by the vector's float32 scale (little endian).
    scale = max|x| / 127 (1 for a zero vector), code = round-half-even(x / scale), all in
    float32; the stored vector is scale * codes."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    rows, d = x.shape
    scale = (np.abs(x).max(axis=1) / np.float32(127.0)).astype(np.float32) if d else np.zeros(rows, np.float32)
    scale[scale == 0] = np.float32(1.0)
    codes = np.clip(np.rint(x / scale[:, None]), -127, 127).astype(np.int8)
    out = np.empty((rows, d + 4), dtype=np.uint8)
    out[:, :d] = codes.view(np.uint8)
    out[:, d:] = scale.view(np.uint8).reshape(rows, 4)
    return out


def quantize_int8_device(x):
    """The same on a torch device tensor: [rows, d] float32 -> [rows, d+4] uint8."""
    import torch
    rows, d = x.shape
    scale = x.abs().amax(dim=1) / 127.0
    scale = torch.where(scale == 0, torch.ones_like(scale), scale)
    codes = torch.clamp(torch.round(x / scale[:, None]), -127, 127).to(torch.int8)
    out = torch.empty((rows, d + 4), dtype=torch.uint8, device=x.device)
    out[:, :d] = codes.view(torch.uint8)
    out[:, d:] = scale.contiguous().view(torch.uint8).reshape(rows, 4)
    return out


@functools.lru_cache(maxsize=4)
def pq_codebooks(w: Workload) -> np.ndarray:
    """[pq_m, 256, d/pq_m] float32 codebooks for "pq8" storage (data preparation: the
    library takes them as given, like the centroids).  Not trained: codeword c of every
    subspace is the matching slice of the c-th of 256 vectors drawn from the mixture with
    the recipe of the stored vectors (a k-means initialisation), which is all the search
    path needs — it is exact over whatever the codes stand for."""
    assert w.storage == "pq8" and w.pq_m > 0 and w.d % w.pq_m == 0
    cen = centroids(w)
    rng = _rng(w, _STREAM_CODEBOOK)
    comp = rng.integers(0, w.nlist, size=256)
    x = cen[comp] + np.float32(w.sigma) * rng.standard_normal((256, w.d), dtype=np.float32)
    x /= np.linalg.norm(x, axis=1, keepdims=True)
    dsub = w.d // w.pq_m
    return np.ascontiguousarray(x.astype(np.float32).reshape(256, w.pq_m, dsub).transpose(1, 0, 2))


def pq_encode_host(x: np.ndarray, codebooks: np.ndarray) -> np.ndarray:
    """Data preparation for "pq8" storage: [rows, d] float32 -> [rows, M] uint8, code m =
    the codeword of subspace m nearest to the vector's slice in Euclidean distance
    (ties to the smaller code), computed in float32 as argmin of |c|^2 - 2 <x_m, c>."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    M, _, dsub = codebooks.shape
    out = np.empty((x.shape[0], M), dtype=np.uint8)
    for m in range(M):
        cb = codebooks[m]
        cost = (cb * cb).sum(axis=1)[None, :] - np.float32(2.0) * (x[:, m * dsub:(m + 1) * dsub] @ cb.T)
        out[:, m] = np.argmin(cost, axis=1).astype(np.uint8)
    return out


def pq_encode_device(x, codebooks_dev, rows_per_step: int = 32768):
    """The same on a torch device tensor [rows, d] float32 -> [rows, M] uint8 (batched over
    the subspaces, a slab of rows at a time so that the cost matrix stays small)."""
    import torch
    M, _, dsub = codebooks_dev.shape
    rows = x.shape[0]
    out = torch.empty((rows, M), dtype=torch.uint8, device=x.device)
    c2 = (codebooks_dev * codebooks_dev).sum(dim=2)                       # [M, 256]
    cbt = codebooks_dev.transpose(1, 2).contiguous()                      # [M, dsub, 256]
    for r0 in range(0, rows, rows_per_step):
        xs = x[r0:r0 + rows_per_step].reshape(-1, M, dsub).transpose(0, 1)     # [M, rows, dsub]
        cost = c2[:, None, :] - 2.0 * torch.bmm(xs, cbt)                       # [M, rows, 256]
        out[r0:r0 + rows_per_step] = torch.argmin(cost, dim=2).transpose(0, 1).to(torch.uint8)
    return out


def split_int8_records(rec: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """[rows, d+4] uint8 records -> (codes [rows, d] int8, scales [rows] float32)."""
    rec = np.ascontiguousarray(rec, dtype=np.uint8)
    d = rec.shape[1] - 4
    return rec[:, :d].view(np.int8), np.ascontiguousarray(rec[:, d:]).view(np.float32).reshape(-1)


def _group_rows(w: Workload, off: np.ndarray, group: int) -> Tuple[int, int, int, int]:
    l0 = group * GROUP
    l1 = min(w.nlist, l0 + GROUP)
    return l0, l1, int(off[l0]), int(off[l1])


def group_vectors_host(w: Workload, cen: np.ndarray, off: np.ndarray, group: int) -> np.ndarray:
    """Row-major vectors of the lists of one group, list after list, in the
    storage type (float32, float16, or int8 records), drawn with NumPy."""
    l0, l1, r0, r1 = _group_rows(w, off, group)
    rows = r1 - r0
    g = _rng(w, _STREAM_NOISE, group).standard_normal((rows, w.d), dtype=np.float32)
    label = np.repeat(np.arange(l0, l1), np.diff(off[l0:l1 + 1]))
    x = cen[label] + np.float32(w.sigma) * g
    x /= np.linalg.norm(x, axis=1, keepdims=True)
    if w.storage == "int8":
        return quantize_int8_host(x)
    if w.storage == "pq8":
        return pq_encode_host(x, pq_codebooks(w))
    return x.astype(np.float16 if w.storage == "fp16" else np.float32)


def group_vectors_device(w: Workload, cen_dev, off: np.ndarray, group_begin: int, group_end: int,
                         device="cuda"):
    """Same recipe on the GPU with torch's generator; returns a device tensor
    [rows, d] covering groups [group_begin, group_end), list-major."""
    import torch
    parts = []
    gen = torch.Generator(device=device)
    cb_dev = torch.from_numpy(pq_codebooks(w)).to(device) if w.storage == "pq8" else None
    for group in range(group_begin, group_end):
        l0, l1, r0, r1 = _group_rows(w, off, group)
        rows = r1 - r0
        gen.manual_seed(_torch_seed(w, _STREAM_NOISE, group))
        g = torch.randn((rows, w.d), generator=gen, device=device, dtype=torch.float32)
        sizes = torch.from_numpy(np.diff(off[l0:l1 + 1])).to(device)
        label = torch.repeat_interleave(torch.arange(l0, l1, device=device), sizes)
        g.mul_(w.sigma).add_(cen_dev[label])
        g.div_(torch.linalg.vector_norm(g, dim=1, keepdim=True))
        parts.append(quantize_int8_device(g) if w.storage == "int8" else
                     pq_encode_device(g, cb_dev) if w.storage == "pq8" else
                     g.to(torch.float16) if w.storage == "fp16" else g)
    return torch.cat(parts, dim=0) if len(parts) != 1 else parts[0]


def user_ids_host(w: Workload) -> np.ndarray:
    """[n] int64: the user id of the vector at each list-major position."""
    return _rng(w, _STREAM_IDS).permutation(w.n).astype(np.int64)


def user_ids_device(w: Workload, device="cuda"):
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(_torch_seed(w, _STREAM_IDS, 0))
    return torch.randperm(w.n, generator=gen, device=device, dtype=torch.int64)


def list_labels(off: np.ndarray) -> np.ndarray:
    """[n] int32 list number of every list-major position."""
    return np.repeat(np.arange(len(off) - 1, dtype=np.int32), np.diff(off))


@dataclass
class HostIndex:
    """A whole index in host memory (small configurations)."""
    w: Workload
    centroids: np.ndarray   # [nlist, d] float32
    vectors: np.ndarray     # [n, d] float32 or float16, list-major
    ids: np.ndarray         # [n] int64
    offsets: np.ndarray     # [nlist+1] int64


def build_host_index(w: Workload) -> HostIndex:
    cen = centroids(w)
    off = list_offsets(w)
    parts = [group_vectors_host(w, cen, off, g) for g in range(w.ngroups)]
    vec = np.ascontiguousarray(np.concatenate(parts, axis=0))
    return HostIndex(w, cen, vec, user_ids_host(w), off)


def iter_device_chunks(w: Workload, cen_dev, off: np.ndarray, groups_per_chunk: int,
                       device="cuda") -> Iterator[Tuple[int, int, "object"]]:
    """Yields (list_begin, list_end, vectors[rows, d]) covering the index in
    list order, a few groups at a time, so that a caller can hand the index to
    the library without ever holding all of it."""
    for g0 in range(0, w.ngroups, groups_per_chunk):
        g1 = min(w.ngroups, g0 + groups_per_chunk)
        yield g0 * GROUP, min(w.nlist, g1 * GROUP), group_vectors_device(w, cen_dev, off, g0, g1, device)
