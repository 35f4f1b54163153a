/*
 * ivf.h — C ABI of the MI355X (gfx950) batched IVF inner-product top-k retrieval
 * library: the retrieval stage of a decoupled retrieve-then-generate RAG pipeline.
 *
 * The operation: for a batch of query embeddings, match them against the stored
 * chunk embeddings by similarity search and return the k most relevant chunks per
 * query (paper Section 2.2 "On-demand RAG Serving"; one batch per call, Section 2.3
 * "Batch Scheduling"; top-k, Section 6.1 "Workloads"; results never approximated,
 * Section 6.1 "Key Metrics").  Only part of the store needs to live in the fast
 * memory tier; the rest is loaded on demand per retrieval batch (Section 4.2
 * "Database partitions"; Section 5 "Lazy dynamic transfer") — here the fast tier is
 * HBM and the slow tier is pinned host memory.  Index type and metric are fixed by
 * the benchmark, not by the paper: IVF-Flat, inner product, given centroids.
 *
 * Conventions
 *   - Every function returns 0 on success or a negative ivf_status; it never aborts
 *     and never throws.  ivf_last_error() gives a thread-local message for the last
 *     failing call on the calling thread.
 *   - "host or device" pointers are classified by the library itself.
 *   - The library COPIES what it is given at upload; the caller keeps ownership of
 *     its buffers and may free them when the call returns.
 *   - One search (or upload, or budget change) at a time per index: calls on the
 *     same index must not overlap on the host.  On the device, consecutive searches of
 *     an index share scratch memory; the library orders them itself (a search issued on
 *     another stream than the one before it starts behind that one), so any stream may
 *     be passed to any call.  Different indexes are independent.
 *   - Limits: d a multiple of 8 (16 for IVF_INT8) and d <= 4096; 1 <= k <= 1024;
 *     1 <= nprobe <= 1024 (nprobe above nlist is clamped to nlist); nq <= 65535 per
 *     call; n < 2^32; nlist < 2^28; a list holds at most 65535 * 64 vectors.
 *   - Ordering rule: best first by (score descending, user id ascending, upload
 *     position ascending).  The GPU accumulates scores in fp32.
 */
#ifndef IVF_H
#define IVF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ivf_index ivf_index; /* opaque, owned by the library */

typedef enum {
    IVF_OK = 0,
    IVF_ERR_INVALID = -1,   /* null pointer, bad size, call out of sequence */
    IVF_ERR_OOM_DEVICE = -2,
    IVF_ERR_OOM_HOST = -3,  /* pinned host memory */
    IVF_ERR_HIP = -4,       /* a HIP runtime call failed; message has hipGetErrorString */
    IVF_ERR_LIMIT = -5      /* argument beyond a documented limit */
} ivf_status;

/*
 * Storage types of the list data.  IVF_INT8 is the compressed form (the paper points at
 * quantised / on-disk indexes as the way to trade memory for accuracy, Section 6.5
 * "On-Disk Index", without fixing a format; this one is the build's own): each stored
 * vector is a record of d signed 8-bit codes followed by one fp32 scale (d+4 bytes, little
 * endian, d a multiple of 16) and stands for the vector scale*codes, so that
 *     score(q, i) = scale_i * sum_t q_t * code_{i,t}        (fp32 accumulate)
 * exactly as for the other types but over 1 byte per dimension.  Quantising the
 * embeddings (choice of scale, rounding) is data preparation by the caller, like the
 * assignment to lists: the search is exact over the vectors the records stand for.
 */
enum { IVF_FP32 = 0, IVF_FP16 = 1, IVF_INT8 = 2, IVF_PQ8 = 3 };

/*
 * IVF_PQ8: lists of product-quantisation codes, the kind of code the paper's on-disk index
 * variant keeps in memory (Section 6.5 "On-Disk Index"; the paper fixes no format, this one
 * is the build's own).  The d dimensions are cut into m subspaces of d/m consecutive
 * dimensions; subspace j has a codebook of 256 codewords; a stored vector is m one-byte
 * codes and stands for the concatenation of the codewords they select, so that
 *     score(q, i) = sum_j <q_j, codebook[j][code_ij]>        (fp32, ascending j)
 * Training the codebooks and encoding the embeddings are data preparation by the caller,
 * like the centroids and the assignment to lists: the search is exact over the vectors
 * the codes stand for.
 *   codebooks  [m, 256, d/m] fp32, host or device; copied.  m a multiple of 16, m <= 128,
 *              d a multiple of m.
 * Call it before an upload with dtype IVF_PQ8 (whose `vectors` are then [n, m] bytes); the
 * codebooks stay until they are set again.  Host-resident code lists are read in place
 * only (ivf_search returns IVF_ERR_INVALID in the staged mode, "host_direct" = 0).
 */
int ivf_index_set_pq_codebooks(ivf_index *idx, int d, int m, const float *codebooks);

/* Creates an empty index bound to the current HIP device. */
int ivf_index_create(ivf_index **out);

/* Frees device and pinned-host memory of the index.  NULL is allowed. */
void ivf_index_destroy(ivf_index *idx);

/*
 * ivf_index_upload — hand a complete IVF-Flat index to the library (data preparation,
 * not part of the timed path).  Vectors are ALREADY grouped by inverted list.
 *   d             embedding dimension
 *   nlist         number of inverted lists (= number of centroids)
 *   n             number of stored vectors
 *   centroids     [nlist, d] fp32 row-major, host or device
 *   vectors       [n, d] row-major in list order, fp32 or IEEE binary16 per `dtype`
 *                 (IVF_INT8: [n] records of d+4 bytes, IVF_PQ8: [n, m] code bytes, see
 *                 above), host or device
 *   ids           [n] user ids in the same order, host or device
 *   list_offsets  [nlist+1], list j owns rows [list_offsets[j], list_offsets[j+1]);
 *                 list_offsets[0] = 0, list_offsets[nlist] = n; host or device
 * The library re-lays the vectors out for its scan kernel.  Everything starts
 * HBM-resident.  Replaces any previous content of the index.
 */
int ivf_index_upload(ivf_index *idx, int d, int64_t nlist, int64_t n, const float *centroids,
                     const void *vectors, int dtype, const int64_t *ids,
                     const int64_t *list_offsets);

/*
 * The same upload in pieces, for indexes too large for the caller to hold next to
 * the library's copy: begin (sizes, centroids, list table), then any number of
 * upload_lists calls that together cover lists [0, nlist) in ascending order without
 * gaps, then end (builds the id tables).  `vectors`/`ids` of a piece cover rows
 * [list_offsets[list_begin], list_offsets[list_end]) only.
 */
int ivf_index_upload_begin(ivf_index *idx, int d, int64_t nlist, int64_t n,
                           const float *centroids, int dtype, const int64_t *list_offsets);
int ivf_index_upload_lists(ivf_index *idx, int64_t list_begin, int64_t list_end,
                           const void *vectors, const int64_t *ids);
int ivf_index_upload_end(ivf_index *idx);

/*
 * ivf_set_device_budget — bytes of HBM the list data may occupy (the analogue of the
 * number of resident database partitions, Section 4.2).  Lists are ranked by
 * (length descending, list number ascending) and stay HBM-resident, in that order,
 * while their padded size still fits in `bytes`; all others are moved to pinned host
 * memory and cross PCIe once per search batch that probes them.  Two ways, chosen with
 * ivf_set_option("host_direct", ...):
 *   1 (default)  the scan kernel reads them in place from pinned host memory, in the same
 *                launch as the HBM-resident lists (measured ~56 GB/s, 97 % of the box's
 *                pinned host-to-device copy rate);
 *   0            they are copied with hipMemcpyAsync on side streams into a ring of
 *                staging buffers ("stage_mb", "nstage"), neighbouring lists merged into
 *                one copy, the copies of a chunk spread over "nside" copy streams (a copy
 *                of one ~2 MB list is too short to reach the link's rate by itself), and
 *                each chunk is scanned on the caller's stream as soon as its events fire,
 *                while the resident lists are scanned meanwhile (measured 54 GB/s, 94 % of
 *                the copy rate, with four copy streams; 42 GB/s with one).  This is the
 *                fallback for systems where device kernels cannot read host memory.
 * INT64_MAX (or anything at least the index size) makes everything resident again.
 * Results of ivf_search do not depend on the budget or on the mode.
 *
 * The call may be repeated at any time between searches (the paper changes the number of
 * resident partitions between retrieval batches, Sections 4.2 and 5): only the lists that
 * change tier are copied across PCIe.  List data lives in pools of segments (a sixteenth
 * of the index each, between 64 MiB and "segment_mb", default 2048); after evictions the
 * least-filled HBM segments are emptied into the holes of the others with device-to-device
 * copies and freed, so the HBM actually held (ivf_info.device_pool_bytes) follows the
 * budget to within about one segment and no second copy of a tier ever exists.
 * ivf_set_option("residency_policy", 1) ranks lists by how often they have been probed so
 * far (then length, then number) instead of by length.  Blocks until the move is done.
 * If memory runs out half-way the lists moved so far stay where they are (every list
 * always has exactly one valid place) and the error is returned.
 */
int ivf_set_device_budget(ivf_index *idx, int64_t bytes);

/*
 * ivf_set_device_budget_async — the same change of residency, carried out in the
 * background while searches go on (the paper adjusts the resident partitions lazily,
 * during the retrieval phase, on a stream of its own and synchronises only when needed:
 * Section 5).  The call waits for the searches issued so far, works out which lists change
 * tier, issues the first copies on the library's move stream and returns.  Lists move in
 * batches ("move_chunk_kb", default 65536; at most "move_inflight_kb", default 4194304,
 * under way at once), in three phases: evictions (least valuable list first), compaction
 * of the HBM pool, loads (most valuable first).  A list keeps being searched at its old
 * place until its copy has landed and the updated address table has reached the device
 * behind all earlier searches; the old place is released only after those searches have
 * finished, so every search sees each list in exactly one valid place and results never
 * depend on how far the change has got.  The change advances inside every ivf_search,
 * ivf_budget_progress and ivf_budget_wait call (nothing runs on a thread of the
 * library's own); freeing an emptied segment waits for the device.
 *   ivf_budget_progress  non-blocking step; reports the lists (and their padded bytes) that
 *                        still have to change tier and whether anything is outstanding
 *                        (pointers may be NULL)
 *   ivf_budget_wait      blocks until the change is complete
 * A change that runs out of memory stops where it is (searches stay correct); progress
 * and wait then return the error until the next budget call.  Calling either budget
 * function during a change lets the copies under way finish, drops the rest and plans
 * anew from the placement reached.  Like searches, these calls must not overlap other
 * calls on the same index.
 */
int ivf_set_device_budget_async(ivf_index *idx, int64_t bytes);
int ivf_budget_progress(ivf_index *idx, int64_t *pending_lists, int64_t *pending_bytes, int *busy);
int ivf_budget_wait(ivf_index *idx);

/*
 * ivf_search — batched top-k inner-product search.
 *   queries     [nq, d] fp32 row-major: a DEVICE pointer, or pinned host memory
 *               (hipHostMalloc).  Pinned queries are first copied to scratch memory on
 *               the stream of the search's first kernel (for ivf_search_queued that is
 *               a stream of the library, so the copy does not queue behind the caller's
 *               stream); they must stay unchanged until the search is done.  Pageable
 *               host memory is refused (IVF_ERR_INVALID).
 *   nq          batch size (0 is allowed and does nothing)
 *   nprobe      inverted lists scanned per query (the nprobe largest <q, centroid>,
 *               ties to the smaller list number)
 *   k           results per query
 *   out_ids     [nq, k] int64 DEVICE pointer: user ids, best first; -1 where fewer
 *               than k candidates exist
 *   out_scores  [nq, k] fp32 DEVICE pointer: inner products; -inf where padded
 *               (both are only written, by the final selection kernel, so pinned host
 *               memory works as well and saves the copy back: the retrieval worker does
 *               that)
 *   stream      hipStream_t (NULL = default stream).  Work is enqueued on it; the
 *               outputs are valid once the caller has synchronised it.  The call does
 *               not block once the scratch buffers are large enough, except in the
 *               staged host-list mode ("host_direct" = 0), where it blocks until the
 *               copies of the probed host-resident lists have been issued (one internal
 *               side stream, joined to `stream` with events).
 * The first call (and any call with a larger nq*nprobe or k than before) allocates
 * scratch memory; later calls reuse it.
 */
int ivf_search(ivf_index *idx, const float *queries, int64_t nq, int nprobe, int k,
               int64_t *out_ids, float *out_scores, void *stream);

/*
 * ivf_search_queued — the same search for callers that queue searches back to back (a
 * serving loop, the retrieval worker): results are identical to ivf_search's, but the
 * stages of consecutive searches overlap.  The paper keeps its accelerator busy by
 * starting the next items on streams of their own while the current one is still being
 * worked on (Section 4.3 "LLM Prefetching Pipeline"); here the coarse quantisation, probe
 * selection and regrouping of search i+1 run under the list scan of search i, and the
 * final selection of search i (on the caller's stream) under the scan of search i+1.  The
 * library uses three streams of its own (two for the front stages, one for the scans) and
 * three sets of scratch memory taken in turn.  A process has four hardware queues, and
 * streams that share one run one after the other whatever their events say, so the three
 * must sit on queues other than the caller's and each other's; HIP does not tell which
 * queue a stream got.  The first queued search of an index that finds `stream` idle
 * therefore tries it out (once per index, a few milliseconds, with a device-wide
 * synchronisation): it makes streams one by one, runs a 60 us kernel on one stream and
 * an empty one on the other, keeps a stream if the empty kernel ends first against the
 * caller's stream and every stream kept so far, and destroys the others.  A caller that
 * changes streams later keeps that choice.  The library makes its streams when they are
 * first needed (these three, the copy streams of the staged mode, those of a budget
 * change), so an index that never uses a feature adds no stream to the process.
 *   queries_ready  hipEvent_t after which `queries` may be read, or NULL if it may be
 *                  read as soon as the call is made.  Unlike ivf_search, the call does NOT
 *                  order its reading of `queries` behind earlier work on `stream`: that
 *                  is what lets it start under the previous search.  `queries` must stay
 *                  unchanged until the search is done.
 *   stream         the final selection runs on it, behind the scan: the outputs are valid
 *                  once the caller has synchronised it, and work the caller queued on it
 *                  before the call (say, a copy out of out_ids) precedes the writes to
 *                  out_ids / out_scores.
 * While a budget change is under way, while any list is host-resident (the scan is then
 * bound by PCIe and nothing is gained), with timing level 1, on a capturing stream, and
 * when the lists to scan are bounded by less than "queue_min_mb" MiB (default 256: the
 * overlap cannot repay a dozen extra stream and event calls) the search runs exactly like
 * ivf_search, behind queries_ready.  Everything else is as for ivf_search: same
 * limits, same scratch growth on first use (of each of the three sets).  Pass a stream
 * of your own rather than the legacy default stream (NULL), whose implicit
 * synchronisation with other streams costs most of the overlap.
 */
int ivf_search_queued(ivf_index *idx, const float *queries, int64_t nq, int nprobe, int k,
                      int64_t *out_ids, float *out_scores, void *stream, void *queries_ready);

/*
 * ivf_search_noalloc — ivf_search for callers that cannot allocate device memory: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels and bit-identical results, but the search scratch (coarse
 * scores, probe tables, scan items, score blocks) is carved from a static device array
 * of 64 MiB inside the library instead of being allocated on first use; the call never
 * allocates or frees memory.  Each GPU on which the library creates an index holds its
 * own copy of that array until the process ends.
 *   - A search that needs more returns IVF_ERR_LIMIT with the size in the message; the
 *     need is about 4*nq*nlist bytes plus 292 bytes per 64-vector block of nq times the
 *     nprobe longest lists, plus 4*nq*d for queries in pinned host memory (the benchmark's 100k, 2M and 20M-vector configurations fit,
 *     the 100M one with 128 queries does not).
 *   - IVF_ERR_INVALID while a budget change is under way (it allocates and frees pool
 *     segments) and in the staged host-list mode ("host_direct" = 0: staging buffers);
 *     host-resident lists read in place are fine.
 *   - The array is shared by every index on the GPU and keeps the last call's contents
 *     (what must start at zero is cleared by the search itself); two calls that overlapped
 *     on one GPU would race on it.  Calls issued one after
 *     the other are ordered on the device by the library, whatever their streams and
 *     indexes; calls that overlap on one GPU from several host threads are serialised by
 *     a lock while they are issued, but the introspection calls (ivf_debug_last_*,
 *     ivf_last_search_stats) then read whatever search used the array last.
 */
int ivf_search_noalloc(ivf_index *idx, const float *queries, int64_t nq, int nprobe, int k,
                       int64_t *out_ids, float *out_scores, void *stream);

/* Thread-local message of the last error on this thread ("" if none). */
const char *ivf_last_error(void);

/* ---- introspection (evidence and tests; not on the hot path) ---- */

typedef struct {
    int32_t d, dtype;
    int64_t nlist, n;
    int64_t max_list_len;
    int64_t index_bytes;        /* padded list data, device + host */
    int64_t device_list_bytes;  /* padded list data resident in HBM */
    int64_t host_list_bytes;    /* padded list data in pinned host memory */
    int64_t resident_lists;
    int64_t scratch_bytes;      /* search scratch currently allocated */
    int64_t device_pool_bytes;  /* HBM held by the list pool (whole segments, >= device_list_bytes) */
    int64_t host_pool_bytes;    /* pinned host memory held by the list pool */
    int64_t moved_h2d_bytes;    /* last budget change (so far, if under way): bytes copied host -> HBM, */
    int64_t moved_d2h_bytes;    /*   HBM -> host, */
    int64_t moved_d2d_bytes;    /*   and inside HBM while compacting the pool */
} ivf_info;
int ivf_get_info(ivf_index *idx, ivf_info *out);

/* Probed lists of the last search, best first: [nq, nprobe] int32 DEVICE pointer,
   copied on `stream`. */
int ivf_debug_last_probes(ivf_index *idx, int32_t *out_lists, void *stream);

/* Coarse scores <q, centroid> of the last search: [nq, nlist] fp32 DEVICE pointer,
   copied on `stream` (stage-wise parity of the coarse quantiser). */
int ivf_debug_last_coarse(ivf_index *idx, float *out_scores, void *stream);

/* Reads list `list` back from the library's own storage (HBM or pinned host) into
   row-major HOST buffers: out_vectors [len, d] in the index dtype, out_ids [len].
   Either may be NULL.  Returns the list length through *len. */
int ivf_debug_read_list(ivf_index *idx, int64_t list, void *out_vectors, int64_t *out_ids,
                        int64_t *len);

typedef struct {
    int64_t unique_lists;        /* distinct lists probed by the batch */
    int64_t pairs;               /* (query, list) pairs = nq * nprobe */
    int64_t scanned_vectors;     /* sum of len over unique probed lists */
    int64_t scan_bytes;          /* the same in bytes of stored data (unpadded) */
    int64_t scan_bytes_resident; /* part of scan_bytes read from HBM-resident lists */
    int64_t scan_bytes_streamed; /* part copied from pinned host memory for this batch */
    int64_t scan_items;          /* 64-vector work items launched */
} ivf_search_stats;
/* Statistics of the last search; synchronises the stream it ran on. */
int ivf_last_search_stats(ivf_index *idx, ivf_search_stats *out);

/* Stage timing with HIP events on the search's own stream.  Level 1: every search
   records events around all its stages; level 2: only around the scan and the streaming
   of host lists (three event records instead of seven, which matters for searches that
   take ~100 us; the other stages then read 0 and TOTAL covers the two); 0: off.  The
   events of the last 64 searches are kept; ivf_get_stage_ms waits for the search `back`
   calls ago (0 = the last one) and returns its stage times in milliseconds. */
enum {
    IVF_STAGE_COARSE = 0,   /* centroid GEMM + tile maxima */
    IVF_STAGE_PROBE = 1,    /* top-nprobe selection */
    IVF_STAGE_REGROUP = 2,  /* list-major regrouping + work plan */
    IVF_STAGE_SCAN = 3,     /* scan of HBM-resident lists (one kernel launch) */
    IVF_STAGE_STREAM = 4,   /* host-resident lists: copies + their scans (0 if none) */
    IVF_STAGE_SELECT = 5,   /* final k-selection */
    IVF_STAGE_TOTAL = 6,
    IVF_NUM_STAGES = 7
};
int ivf_set_timing(ivf_index *idx, int level);
int ivf_get_stage_ms(ivf_index *idx, int back, float *ms /* [IVF_NUM_STAGES] host */);

/* A plain copy kernel over `bytes` bytes (multiple of 16) of DEVICE memory, enqueued on
   `stream`: reads `bytes`, writes `bytes`, nothing else.  It is the reference point of
   known size against which hardware byte counters of the search kernels are scaled. */
int ivf_debug_copy(void *dst, const void *src, int64_t bytes, void *stream);

/* A plain streaming read of `bytes` bytes (multiple of 98304) of DEVICE memory with the
   scan kernel's access pattern and no arithmetic: its rate is the practical ceiling of
   the list scan on the machine at hand.  `sink` is a DEVICE word that is not written
   for ordinary data. */
int ivf_debug_read(const void *src, int64_t bytes, void *sink, void *stream);

/* Tuning knobs; unknown names or values return IVF_ERR_INVALID.  Defaults are the tuned
   values.  "host_direct" 0|1 (see ivf_set_device_budget), "stage_mb" 1..4096, "nstage"
   2..8, "nside" 1..4 (copy streams of the staged mode: the copies of a chunk go round
   them), "scan_unroll" 8|16 (16-byte
   loads per lane and register buffer), "scan_waves" 1|2|4|8 (wavefronts per workgroup),
   "scan_split" 0|1|2|4 (wavefronts that share one 64-vector block, each taking a slice of the
   dimensions; 0 = as many as leave each a share of 48 KiB, fixed per index; partial sums are
   added in LDS, so scores may differ in the last bit between settings), "queue_min_mb" (see
   ivf_search_queued), "queue_fronts" 0|1|2 (streams that the front stages of queued searches
   alternate between; 0 = two behind short scans, one behind long ones),
   "scan_prune" 0|1|2 (store pruning off / on for large plans of flat and int8 lists / always, also
   over product-quantisation codes, where it costs more than it saves),
   "regroup_fused" 0|1 (1 = searches with at most 1024 lists and 2048 (query, list) pairs
   regroup in a single launch), "sel_threads" 0|256|1024 (workgroup size of the selection kernels; 0 = by problem size),
   "residency_policy" 0|1 and "segment_mb" (see ivf_set_device_budget; the segment size
   applies from the next upload), "move_chunk_kb" and "move_inflight_kb" (see
   ivf_set_device_budget_async). */
int ivf_set_option(ivf_index *idx, const char *name, int64_t value);

/* ---- batch-size choice for the retrieval worker (host arithmetic, no GPU) ----
 *
 * Backlog-aware batch scheduling (paper Section 4.4, Eq. 4-8).  T(B) = a * B^c models
 * the time of one ivf_search over a batch of B queries; with n requests queued, k equal
 * batches served in turn give an average latency of (k+1)/2 * T(n/k) - mean arrival time
 * (Eq. 5 for k = 1, Eq. 6); one batch is at least as good as k batches iff
 * 2 k^c <= k+1 (Eq. 7; c <= log2(3/2) for k = 2, Eq. 8).
 */

/* Least-squares fit of log T = log a + c log B to m >= 1 measured samples (all > 0);
   m = 1 or equal batch sizes give c = 0. */
int ivf_sched_fit(const double *batch_sizes, const double *times, int m, double *a, double *c);

/* T(B) = a * B^c. */
double ivf_sched_batch_time(double a, double c, double batch_size);

/* Average latency of n queued requests served as k equal batches (Eq. 5, 6);
   mean_arrival = (1/n) sum t_i, in the unit of a. */
int ivf_sched_avg_latency(double a, double c, int64_t n, int64_t k, double mean_arrival, double *latency);

/* 1 if one batch is at least as good as k equal batches (Eq. 7), 0 if not, < 0 on error. */
int ivf_sched_single_batch_is_best(double c, int64_t k);

/* Scores every candidate batch size for a queue of n requests and returns the best
   (ties to the larger batch).  A candidate B < n is served as floor(n/B) batches of B and
   then one batch of the r requests left over, which takes T(r); a request waits until its
   batch is done, which gives Eq. 6 when B divides n; a candidate >= n is one batch of n
   (Eq. 5).  best_latency may be NULL. */
int ivf_sched_choose(double a, double c, int64_t n, const int64_t *candidates, int m, double mean_arrival,
                     int64_t *best_batch, double *best_latency);

/* ---- retrieval worker: request queue -> batches -> context queue ----
 *
 * The retrieval half of the decoupled pipeline (paper Section 4.1): requests are put in
 * a retrieval queue; a worker thread forms batches on its own, runs ivf_search on a
 * stream of its own and puts each request's result in a context queue, from which the
 * consumer (the generation side) takes it.  With a backlog of n requests the worker
 * serves them in batches of the size the backlog-aware rule picks (Section 4.4;
 * candidates 1, 2, 4, ... max_batch; T(B) fitted to the worker's own batch timings; the
 * whole backlog up to max_batch until two batch sizes have been timed).
 *
 * While a worker runs it is the only caller of ivf_search on its index (no other
 * search, upload or direct budget change on that index until ivf_worker_stop; budget changes
 * go through ivf_worker_set_device_budget).  Queries and
 * results are HOST buffers; submit and wait may be called from any threads.
 */
typedef struct ivf_worker ivf_worker;

typedef struct {
    int64_t requests_submitted, requests_done, batches, largest_batch;
    int64_t queued;            /* waiting in the retrieval queue right now */
    int64_t results_waiting;   /* finished, not yet taken from the context queue */
    double fit_a_ms, fit_c;    /* last fit of T(B) = a * B^c (0 until there is one) */
    int64_t budget_changes;    /* budget changes taken up by the worker so far */
    int64_t budget_pending_lists;  /* lists that still have to change tier */
    int64_t budget_busy;       /* 1 while a change is under way or asked for */
    int64_t resident_lists;    /* as of the worker's last look */
    int64_t budget_error;      /* error code of the last change, 0 if none */
} ivf_worker_stats;

/* Starts the worker thread on the current HIP device for searches with (nprobe, k). */
int ivf_worker_start(ivf_index *idx, int nprobe, int k, int max_batch, ivf_worker **out);

/* Copies one query [d] fp32 from HOST memory into the retrieval queue; *ticket names it. */
int ivf_worker_submit(ivf_worker *w, const float *query, uint64_t *ticket);

/* Takes the result of `ticket` out of the context queue into HOST buffers ids[k],
   scores[k].  timeout_ms < 0 waits; otherwise returns 1 if it is not ready in time.
   Every ticket can be taken exactly once (a second take returns IVF_ERR_INVALID). */
int ivf_worker_wait(ivf_worker *w, uint64_t ticket, int64_t *out_ids, float *out_scores, int timeout_ms);

int ivf_worker_get_stats(ivf_worker *w, ivf_worker_stats *out);

/* Asks the worker to change the device budget of its index (the scheduler of the paper
   changes the number of resident partitions while the pipeline runs, Sections 4.2 and 5).
   Returns at once; the worker starts the change between two batches with
   ivf_set_device_budget_async and carries it on while it serves requests (and while it is
   idle), so retrieval never stops for it.  A second request before the first is taken up
   replaces it.  Progress: the budget_* fields of ivf_worker_stats. */
int ivf_worker_set_device_budget(ivf_worker *w, int64_t bytes);

/* Serves what is still queued, stops the thread and frees the worker (results not
   taken are dropped).  Returns the worker's error code if it had failed. */
int ivf_worker_stop(ivf_worker *w);

#ifdef __cplusplus
}
#endif
#endif /* IVF_H */
