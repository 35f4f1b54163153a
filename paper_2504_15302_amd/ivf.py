"""Thin ctypes binding over the C-ABI library (include/ivf.h).  Argument marshalling
only: every step of the search runs in the library's HIP kernels.  There is no CPU
fallback — if the built library is missing, loading fails loudly.

Function names mirror the C entry points: `Index.upload` = ivf_index_upload,
`Index.set_device_budget` = ivf_set_device_budget, `Index.search` = ivf_search, ...
torch is used for device memory and streams only.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libivf_mi355x.so")

IVF_FP32, IVF_FP16, IVF_INT8, IVF_PQ8 = 0, 1, 2, 3
STAGES = ("coarse", "probe", "regroup", "scan", "stream", "select", "total")

EXPORTS = (
    "ivf_index_create", "ivf_index_destroy", "ivf_index_upload", "ivf_index_upload_begin",
    "ivf_index_upload_lists", "ivf_index_upload_end", "ivf_set_device_budget", "ivf_search",
    "ivf_search_queued", "ivf_search_noalloc", "ivf_index_set_pq_codebooks",
    "ivf_set_device_budget_async", "ivf_budget_progress", "ivf_budget_wait", "ivf_worker_set_device_budget",
    "ivf_last_error", "ivf_get_info", "ivf_debug_last_probes", "ivf_debug_last_coarse",
    "ivf_debug_read_list", "ivf_last_search_stats", "ivf_set_timing", "ivf_get_stage_ms",
    "ivf_set_option", "ivf_debug_copy", "ivf_debug_read",
    "ivf_sched_fit", "ivf_sched_batch_time", "ivf_sched_avg_latency", "ivf_sched_single_batch_is_best",
    "ivf_sched_choose",
    "ivf_worker_start", "ivf_worker_submit", "ivf_worker_wait", "ivf_worker_get_stats", "ivf_worker_stop",
)


class IvfError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"ivf error {code}: {msg}")
        self.code = code


class Info(C.Structure):
    _fields_ = [("d", C.c_int32), ("dtype", C.c_int32), ("nlist", C.c_int64), ("n", C.c_int64),
                ("max_list_len", C.c_int64), ("index_bytes", C.c_int64),
                ("device_list_bytes", C.c_int64), ("host_list_bytes", C.c_int64),
                ("resident_lists", C.c_int64), ("scratch_bytes", C.c_int64),
                ("device_pool_bytes", C.c_int64), ("host_pool_bytes", C.c_int64),
                ("moved_h2d_bytes", C.c_int64), ("moved_d2h_bytes", C.c_int64),
                ("moved_d2d_bytes", C.c_int64)]


class SearchStats(C.Structure):
    _fields_ = [("unique_lists", C.c_int64), ("pairs", C.c_int64), ("scanned_vectors", C.c_int64),
                ("scan_bytes", C.c_int64), ("scan_bytes_resident", C.c_int64),
                ("scan_bytes_streamed", C.c_int64), ("scan_items", C.c_int64)]


class WorkerStats(C.Structure):
    _fields_ = [("requests_submitted", C.c_int64), ("requests_done", C.c_int64), ("batches", C.c_int64),
                ("largest_batch", C.c_int64), ("queued", C.c_int64), ("results_waiting", C.c_int64),
                ("fit_a_ms", C.c_double), ("fit_c", C.c_double),
                ("budget_changes", C.c_int64), ("budget_pending_lists", C.c_int64), ("budget_busy", C.c_int64),
                ("resident_lists", C.c_int64), ("budget_error", C.c_int64)]


_lib = None


def load_library() -> C.CDLL:
    """Loads the built HIP library; raises if it has not been built
    (python -m paper_2504_15302_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2504_15302_amd.build` "
            "(there is no CPU fallback)")
    # torch ships its own HIP runtime under the same SONAME.  Import it first so that
    # the library binds to the runtime torch already loaded: two HIP runtimes in one
    # process do not both see the GPU.
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    vp, i64, i32 = C.c_void_p, C.c_int64, C.c_int
    lib.ivf_index_create.argtypes = [C.POINTER(vp)]
    lib.ivf_index_destroy.argtypes = [vp]
    lib.ivf_index_destroy.restype = None
    lib.ivf_index_upload.argtypes = [vp, i32, i64, i64, vp, vp, i32, vp, vp]
    lib.ivf_index_upload_begin.argtypes = [vp, i32, i64, i64, vp, i32, vp]
    lib.ivf_index_upload_lists.argtypes = [vp, i64, i64, vp, vp]
    lib.ivf_index_upload_end.argtypes = [vp]
    lib.ivf_index_set_pq_codebooks.argtypes = [vp, i32, i32, vp]
    lib.ivf_set_device_budget.argtypes = [vp, i64]
    lib.ivf_set_device_budget_async.argtypes = [vp, i64]
    lib.ivf_budget_progress.argtypes = [vp, C.POINTER(i64), C.POINTER(i64), C.POINTER(i32)]
    lib.ivf_budget_wait.argtypes = [vp]
    lib.ivf_worker_set_device_budget.argtypes = [vp, i64]
    lib.ivf_search.argtypes = [vp, vp, i64, i32, i32, vp, vp, vp]
    lib.ivf_search_queued.argtypes = [vp, vp, i64, i32, i32, vp, vp, vp, vp]
    lib.ivf_search_noalloc.argtypes = [vp, vp, i64, i32, i32, vp, vp, vp]
    lib.ivf_last_error.restype = C.c_char_p
    lib.ivf_get_info.argtypes = [vp, C.POINTER(Info)]
    lib.ivf_debug_last_probes.argtypes = [vp, vp, vp]
    lib.ivf_debug_last_coarse.argtypes = [vp, vp, vp]
    lib.ivf_debug_read_list.argtypes = [vp, i64, vp, vp, C.POINTER(i64)]
    lib.ivf_last_search_stats.argtypes = [vp, C.POINTER(SearchStats)]
    lib.ivf_set_timing.argtypes = [vp, i32]
    lib.ivf_get_stage_ms.argtypes = [vp, i32, C.POINTER(C.c_float)]
    lib.ivf_set_option.argtypes = [vp, C.c_char_p, i64]
    lib.ivf_debug_copy.argtypes = [vp, vp, i64, vp]
    lib.ivf_debug_read.argtypes = [vp, i64, vp, vp]
    dbl, pd, pi64 = C.c_double, C.POINTER(C.c_double), C.POINTER(C.c_int64)
    lib.ivf_sched_fit.argtypes = [pd, pd, i32, pd, pd]
    lib.ivf_sched_batch_time.argtypes = [dbl, dbl, dbl]
    lib.ivf_sched_avg_latency.argtypes = [dbl, dbl, i64, i64, dbl, pd]
    lib.ivf_sched_single_batch_is_best.argtypes = [dbl, i64]
    lib.ivf_sched_choose.argtypes = [dbl, dbl, i64, pi64, i32, dbl, pi64, pd]
    lib.ivf_worker_start.argtypes = [vp, i32, i32, i32, C.POINTER(vp)]
    lib.ivf_worker_submit.argtypes = [vp, vp, C.POINTER(C.c_uint64)]
    lib.ivf_worker_wait.argtypes = [vp, C.c_uint64, vp, vp, i32]
    lib.ivf_worker_get_stats.argtypes = [vp, C.POINTER(WorkerStats)]
    lib.ivf_worker_stop.argtypes = [vp]
    for name in EXPORTS:
        if name not in ("ivf_index_destroy", "ivf_last_error", "ivf_sched_batch_time"):
            getattr(lib, name).restype = C.c_int
    lib.ivf_sched_batch_time.restype = dbl
    _lib = lib
    return lib


def _check(rc: int):
    if rc != 0:
        raise IvfError(rc, load_library().ivf_last_error().decode())


def _ptr(a) -> Optional[int]:
    """Address of a NumPy array (host) or torch tensor (host or device)."""
    if a is None:
        return None
    if isinstance(a, np.ndarray):
        assert a.flags["C_CONTIGUOUS"]
        return a.ctypes.data
    assert a.is_contiguous()
    return a.data_ptr()


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def _dtype_code(a) -> int:
    name = str(a.dtype)
    if name.endswith("float32"):
        return IVF_FP32
    if name.endswith("float16"):
        return IVF_FP16
    if name.endswith("uint8"):          # int8 records: d codes + fp32 scale per row
        return IVF_INT8
    raise TypeError(f"vectors must be float32, float16 or uint8 records, got {a.dtype}")


class Index:
    """Owner of one `ivf_index*`."""

    def __init__(self):
        self._lib = load_library()
        h = C.c_void_p()
        _check(self._lib.ivf_index_create(C.byref(h)))
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            self._lib.ivf_index_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- upload
    def set_pq_codebooks(self, codebooks):
        """codebooks: float32 [m, 256, d/m] (NumPy or torch); uploads with dtype IVF_PQ8 follow."""
        m, ncode, dsub = codebooks.shape
        assert ncode == 256 and str(codebooks.dtype).endswith("float32")
        _check(self._lib.ivf_index_set_pq_codebooks(self._h, m * dsub, m, _ptr(codebooks)))

    def upload(self, centroids, vectors, ids, list_offsets, dtype: Optional[int] = None):
        """dtype: by the array type if None (uint8 = int8 records; pass IVF_PQ8 for code bytes)."""
        nlist, d = centroids.shape
        n = vectors.shape[0]
        dt = _dtype_code(vectors) if dtype is None else dtype
        assert dt == IVF_PQ8 or vectors.shape[1] == (d + 4 if dt == IVF_INT8 else d)
        assert ids.shape[0] == n and list_offsets.shape[0] == nlist + 1
        _check(self._lib.ivf_index_upload(self._h, d, nlist, n, _ptr(centroids), _ptr(vectors),
                                          dt, _ptr(ids), _ptr(list_offsets)))

    def upload_begin(self, centroids, n: int, dtype: int, list_offsets):
        nlist, d = centroids.shape
        _check(self._lib.ivf_index_upload_begin(self._h, d, nlist, n, _ptr(centroids), dtype,
                                                _ptr(list_offsets)))

    def upload_lists(self, list_begin: int, list_end: int, vectors, ids):
        _check(self._lib.ivf_index_upload_lists(self._h, list_begin, list_end, _ptr(vectors), _ptr(ids)))

    def upload_end(self):
        _check(self._lib.ivf_index_upload_end(self._h))

    # ---- placement
    def set_device_budget(self, nbytes: int):
        _check(self._lib.ivf_set_device_budget(self._h, int(nbytes)))

    # ---- search
    def set_device_budget_async(self, nbytes: int):
        _check(self._lib.ivf_set_device_budget_async(self._h, int(nbytes)))

    def budget_progress(self):
        """(lists still to change tier, their bytes, busy) after one non-blocking step."""
        pl, pb, busy = C.c_int64(0), C.c_int64(0), C.c_int(0)
        _check(self._lib.ivf_budget_progress(self._h, C.byref(pl), C.byref(pb), C.byref(busy)))
        return pl.value, pb.value, bool(busy.value)

    def budget_wait(self):
        _check(self._lib.ivf_budget_wait(self._h))

    def search(self, queries, nprobe: int, k: int, out_ids=None, out_scores=None, stream=None):
        """queries: float32 tensor [nq, d], CUDA or pinned host memory.  Returns (ids int64
        [nq,k], scores float32 [nq,k]), CUDA tensors unless the caller passes its own (CUDA
        or pinned); valid once `stream` (default: torch's current stream) has been
        synchronised."""
        import torch
        assert (queries.is_cuda or queries.is_pinned()) and queries.dtype == torch.float32 and queries.is_contiguous()
        nq = queries.shape[0]
        if out_ids is None:
            out_ids = torch.empty((nq, k), dtype=torch.int64, device="cuda")
        if out_scores is None:
            out_scores = torch.empty((nq, k), dtype=torch.float32, device="cuda")
        _check(self._lib.ivf_search(self._h, _ptr(queries), nq, nprobe, k, _ptr(out_ids),
                                    _ptr(out_scores), _stream_handle(stream)))
        return out_ids, out_scores

    def search_queued(self, queries, nprobe: int, k: int, out_ids=None, out_scores=None, stream=None,
                      queries_ready=None):
        """ivf_search_queued: as `search`, but `queries` is read as soon as `queries_ready`
        (a torch.cuda.Event, or None = now) allows, not behind earlier work on `stream`."""
        import torch
        assert (queries.is_cuda or queries.is_pinned()) and queries.dtype == torch.float32 and queries.is_contiguous()
        nq = queries.shape[0]
        if out_ids is None:
            out_ids = torch.empty((nq, k), dtype=torch.int64, device="cuda")
        if out_scores is None:
            out_scores = torch.empty((nq, k), dtype=torch.float32, device="cuda")
        ev = None if queries_ready is None else queries_ready.cuda_event
        _check(self._lib.ivf_search_queued(self._h, _ptr(queries), nq, nprobe, k, _ptr(out_ids),
                                           _ptr(out_scores), _stream_handle(stream), ev))
        return out_ids, out_scores

    def search_noalloc(self, queries, nprobe: int, k: int, out_ids, out_scores, stream=None):
        """ivf_search_noalloc: the caller passes every buffer; the library allocates nothing."""
        import torch
        assert (queries.is_cuda or queries.is_pinned()) and queries.dtype == torch.float32 and queries.is_contiguous()
        nq = queries.shape[0]
        assert tuple(out_ids.shape) == (nq, k) and tuple(out_scores.shape) == (nq, k)
        _check(self._lib.ivf_search_noalloc(self._h, _ptr(queries), nq, nprobe, k, _ptr(out_ids),
                                            _ptr(out_scores), _stream_handle(stream)))
        return out_ids, out_scores

    def search_raw(self, queries_ptr, nq, nprobe, k, out_ids_ptr, out_scores_ptr, stream_ptr=None) -> int:
        """The C call with raw addresses, returning the status code (for error-path tests)."""
        return self._lib.ivf_search(self._h, queries_ptr, nq, nprobe, k, out_ids_ptr, out_scores_ptr, stream_ptr)

    # ---- introspection
    def info(self) -> Info:
        out = Info()
        _check(self._lib.ivf_get_info(self._h, C.byref(out)))
        return out

    def last_probes(self, nq: int, nprobe: int, stream=None):
        import torch
        out = torch.empty((nq, nprobe), dtype=torch.int32, device="cuda")
        _check(self._lib.ivf_debug_last_probes(self._h, _ptr(out), _stream_handle(stream)))
        return out

    def last_coarse(self, nq: int, nlist: int, stream=None):
        import torch
        out = torch.empty((nq, nlist), dtype=torch.float32, device="cuda")
        _check(self._lib.ivf_debug_last_coarse(self._h, _ptr(out), _stream_handle(stream)))
        return out

    def read_list(self, list_no: int, d: int, dtype: int):
        ln = C.c_int64()
        _check(self._lib.ivf_debug_read_list(self._h, list_no, None, None, C.byref(ln)))
        if dtype == IVF_PQ8:
            vec = np.empty((ln.value, d), dtype=np.uint8)            # d = code bytes per vector here
        elif dtype == IVF_INT8:
            vec = np.empty((ln.value, d + 4), dtype=np.uint8)
        else:
            vec = np.empty((ln.value, d), dtype=np.float16 if dtype == IVF_FP16 else np.float32)
        ids = np.empty(ln.value, dtype=np.int64)
        _check(self._lib.ivf_debug_read_list(self._h, list_no, _ptr(vec), _ptr(ids), C.byref(ln)))
        return vec, ids

    def last_search_stats(self) -> SearchStats:
        out = SearchStats()
        _check(self._lib.ivf_last_search_stats(self._h, C.byref(out)))
        return out

    def set_timing(self, level):
        """0/False off, 1/True every stage, 2 the scan and streaming stages only."""
        _check(self._lib.ivf_set_timing(self._h, int(level)))

    def stage_ms(self, back: int = 0) -> dict:
        """Stage times (ms) of the timed search `back` calls ago (0 = the last one)."""
        arr = (C.c_float * len(STAGES))()
        _check(self._lib.ivf_get_stage_ms(self._h, back, arr))
        return {name: float(arr[i]) for i, name in enumerate(STAGES)}

    def debug_copy(self, dst, src, stream=None):
        """Plain device-to-device copy kernel of known size (counter calibration)."""
        assert dst.numel() * dst.element_size() == src.numel() * src.element_size()
        _check(self._lib.ivf_debug_copy(_ptr(dst), _ptr(src), src.numel() * src.element_size(),
                                        _stream_handle(stream)))

    def debug_read(self, src, sink, stream=None):
        """Plain streaming-read kernel over `src` (practical HBM read ceiling)."""
        _check(self._lib.ivf_debug_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink),
                                        _stream_handle(stream)))

    def set_option(self, name: str, value: int):
        _check(self._lib.ivf_set_option(self._h, name.encode(), int(value)))


# ---- batch-size choice for the retrieval worker (ivf_sched_*: host arithmetic, no GPU)

def sched_fit(batch_sizes, times):
    """(a, c) of T(B) = a * B**c fitted to measured samples."""
    m = len(batch_sizes)
    bs = (C.c_double * m)(*[float(b) for b in batch_sizes])
    ts = (C.c_double * m)(*[float(t) for t in times])
    a, c = C.c_double(), C.c_double()
    _check_plain(load_library().ivf_sched_fit(bs, ts, m, C.byref(a), C.byref(c)))
    return a.value, c.value


def sched_batch_time(a: float, c: float, batch_size: float) -> float:
    return float(load_library().ivf_sched_batch_time(a, c, batch_size))


def sched_avg_latency(a: float, c: float, n: int, k: int, mean_arrival: float = 0.0) -> float:
    out = C.c_double()
    _check_plain(load_library().ivf_sched_avg_latency(a, c, n, k, mean_arrival, C.byref(out)))
    return out.value


def sched_single_batch_is_best(c: float, k: int) -> bool:
    rc = load_library().ivf_sched_single_batch_is_best(c, k)
    _check_plain(rc if rc < 0 else 0)
    return rc == 1


def sched_choose(a: float, c: float, n: int, candidates, mean_arrival: float = 0.0):
    m = len(candidates)
    cs = (C.c_int64 * m)(*[int(x) for x in candidates])
    best, lat = C.c_int64(), C.c_double()
    _check_plain(load_library().ivf_sched_choose(a, c, n, cs, m, mean_arrival, C.byref(best), C.byref(lat)))
    return best.value, lat.value


def _check_plain(rc: int):
    if rc != 0:
        raise IvfError(rc, "ivf_sched_* / ivf_worker_* call failed (invalid argument, or the worker has failed)")


class Worker:
    """Owner of one `ivf_worker*`: submit host queries, take results by ticket."""

    def __init__(self, index: Index, nprobe: int, k: int, max_batch: int):
        self._lib = load_library()
        self._index = index          # keeps the index alive
        self.k = k
        self.d = index.info().d
        h = C.c_void_p()
        _check_plain(self._lib.ivf_worker_start(index._h, nprobe, k, max_batch, C.byref(h)))
        self._h = h

    def submit(self, query: np.ndarray) -> int:
        q = np.ascontiguousarray(query, dtype=np.float32)
        assert q.shape == (self.d,)
        t = C.c_uint64()
        _check_plain(self._lib.ivf_worker_submit(self._h, q.ctypes.data, C.byref(t)))
        return t.value

    def wait(self, ticket: int, timeout_ms: int = -1):
        """(ids[k], scores[k]) or None if not ready within the timeout."""
        ids = np.empty(self.k, dtype=np.int64)
        scores = np.empty(self.k, dtype=np.float32)
        rc = self._lib.ivf_worker_wait(self._h, ticket, ids.ctypes.data, scores.ctypes.data, timeout_ms)
        if rc == 1:
            return None
        _check_plain(rc)
        return ids, scores

    def set_device_budget(self, nbytes: int):
        """Asks the worker to change its index's device budget in the background."""
        _check_plain(self._lib.ivf_worker_set_device_budget(self._h, int(nbytes)))

    def stats(self) -> WorkerStats:
        out = WorkerStats()
        _check_plain(self._lib.ivf_worker_get_stats(self._h, C.byref(out)))
        return out

    def stop(self):
        if getattr(self, "_h", None):
            h, self._h = self._h, None
            _check_plain(self._lib.ivf_worker_stop(h))

    def __del__(self):
        try:
            self.stop()
        except Exception:
            pass
