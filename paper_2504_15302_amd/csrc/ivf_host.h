// Host-side state of the IVF retrieval library: error reporting, search scratch, and the
// index object behind the opaque handle of include/ivf.h.  Included by ivf_api.hip only.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <deque>
#include <limits>
#include <map>
#include <new>
#include <numeric>
#include <string>
#include <vector>

#include "../../include/ivf.h"
#include "ivf_coarse.h"
#include "ivf_device.h"
#include "ivf_pool.h"
#include "ivf_pq.h"
#include "ivf_regroup.h"
#include "ivf_scan.h"
#include "ivf_select.h"

extern "C" int ivf_internal_sort_pairs(const int64_t* keys_in, int64_t* keys_out,
                                       const uint32_t* vals_in, uint32_t* vals_out, size_t n,
                                       hipStream_t stream);

namespace {

using namespace ivf;

thread_local std::string g_err;

int fail(int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

#define HIP_TRY(expr)                                                                      \
    do {                                                                                   \
        hipError_t e_ = (expr);                                                            \
        if (e_ != hipSuccess) {                                                            \
            (void)hipGetLastError();                                                       \
            return fail(e_ == hipErrorOutOfMemory ? IVF_ERR_OOM_DEVICE : IVF_ERR_HIP,      \
                        "%s failed: %s", #expr, hipGetErrorString(e_));                    \
        }                                                                                  \
    } while (0)

// A stream of the library's own, made at its first use.
inline int need_stream(hipStream_t& s) {
    if (!s) HIP_TRY(hipStreamCreateWithFlags(&s, hipStreamNonBlocking));
    return 0;
}

bool is_device_ptr(const void* p) {
    hipPointerAttribute_t a;
    hipError_t e = hipPointerGetAttributes(&a, p);
    if (e != hipSuccess) {
        (void)hipGetLastError();   // plain host memory is reported as an error
        return false;
    }
    return a.type == hipMemoryTypeDevice || a.type == hipMemoryTypeManaged ||
           a.type == hipMemoryTypeUnified;
}

template <class T>
void dfree(T*& p) {
    if (p) (void)hipFree(p);
    p = nullptr;
}

void* hbm_alloc(size_t bytes) {
    void* p = nullptr;
    if (hipMalloc(&p, bytes) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
    return p;
}
void hbm_free(void* p) { (void)hipFree(p); }
void* pinned_alloc(size_t bytes) {
    void* p = nullptr;
    if (hipHostMalloc(&p, bytes) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
    return p;
}
void pinned_free(void* p) { (void)hipHostFree(p); }

struct Scratch {
    size_t cap_q_nlist = 0, cap_q_ntile = 0, cap_pairs = 0, cap_blocks = 0, cap_stream_items = 0;
    int64_t cap_nlist = 0;
    float* S = nullptr;
    float* tmax = nullptr;
    int32_t* probes = nullptr;
    int* zeroed = nullptr;          // hist[nlist] | cursor[nlist] | queue[16] | counters (8 x u64) | qthr (nq x u64)
    unsigned long long* qthr = nullptr;   // per query: running lower bounds of its k-th best score
    size_t cap_zero_q = 0;
    uint32_t* wg_totals = nullptr;
    uint32_t* pair_start = nullptr;
    uint32_t* sblk_start = nullptr;
    uint32_t* item_start = nullptr;
    unsigned long long* counters = nullptr;
    uint32_t* pair_flat = nullptr;
    uint32_t* pair_of_probe = nullptr;
    ScanItem* items = nullptr;
    ScanItem* stream_items = nullptr;
    float* scores = nullptr;
    float* bmax = nullptr;
    float* pq_tables = nullptr;     // product-quantised lists: [nq][M][256] inner products with the codewords
    float* q_stage = nullptr;       // device copy of queries that the caller keeps in pinned host memory
    size_t cap_q_stage = 0;         // in floats
    size_t cap_pq_q = 0;
    // pinned host mirrors for the streamed path
    int32_t* h_probes = nullptr;
    size_t h_probes_cap = 0;
    ScanItem* h_items = nullptr;
    size_t h_items_cap = 0;
    size_t bytes = 0;
    bool carved = false;            // buffers are slices of one caller-owned region: never freed one by one
    // Recorded behind the last kernel of the last search that used this set, on whatever
    // stream that was: the next search that uses the set starts behind it.  The handle
    // belongs to the index and outlives the buffers.
    hipEvent_t end = nullptr;
    bool end_recorded = false;
};

constexpr int kSets = 3;           // scratch sets that queued searches go round
constexpr int kMaxStage = 8;
constexpr int kMaxSide = 4;
constexpr int kTimingSlots = 64;   // searches whose stage events are kept
constexpr int kEvPerSearch = 7;    // stage boundaries 0..6

// A change of the device budget is a sequence of list moves (HBM -> host, HBM -> HBM while
// the pool is compacted, host -> HBM), copied in batches on a stream of their own while
// searches go on.  A list keeps being read at its old place until its copy has landed and
// the new address table has reached the device; the old place is released only after
// every search that may still read it has finished.
struct Move {
    int32_t l = 0;
    Loc from, to;
    bool placed = false;             // destination already reserved (compaction)
};
struct MoveBatch {
    hipEvent_t landed = nullptr;     // recorded on the move stream behind the batch's copies
    std::vector<Move> moves;
    size_t bytes = 0;
};
struct Limbo {
    hipEvent_t after = nullptr;      // recorded behind the table update that retires the old places
    const void** table = nullptr;    // pinned snapshot of the address table that the update copies
    std::vector<Move> moves;         // their `from` places are released once `after` has completed
};
enum { kPhaseIdle = 0, kPhaseEvict = 1, kPhaseCompact = 2, kPhaseLoad = 3 };

}  // namespace

struct ivf_index {
    int device = 0;
    int cus = 256;
    bool uploading = false, ready = false;
    int d = 0, dtype = 0, es = 4;
    int pq_m = 0, pq_d = 0;                     // codebooks on record (ivf_index_set_pq_codebooks)
    float* d_codebooks = nullptr;               // [pq_m][256][pq_d / pq_m]
    bool pq_lds_set = false;                    // the code scan has been allowed its dynamic LDS
    int64_t nlist = 0, n = 0, next_list = 0;
    size_t row_bytes = 0, block_bytes = 0;      // one stored vector as uploaded; 64 of them, blocked
    int tail_bytes = 0;                         // bytes of a row behind its d elements (int8: the scale)
    int64_t total_blocks = 0, max_len = 0;
    std::vector<int64_t> offsets, blk_off;
    std::vector<int32_t> len, nblk;
    std::vector<int64_t> top_nblk_prefix;       // prefix sums of nblk sorted descending
    std::vector<const char*> dev_ptr, host_ptr; // per list: where its blocks live (derived from loc)
    std::vector<Loc> loc;
    Pool dpool, hpool;
    // device tables
    float* d_centroids = nullptr;
    int64_t* d_offsets = nullptr;
    int32_t* d_len = nullptr;
    int32_t* d_nblk = nullptr;
    const void** d_list_ptr = nullptr;
    int64_t* d_ids_pos = nullptr;      // only while uploading
    int64_t* d_id_sorted = nullptr;
    uint32_t* d_rank_of_pos = nullptr;
    uint32_t* d_hits = nullptr;        // per list: how often it has been probed (residency policy)
    int64_t resident_lists = 0;
    int64_t moved_h2d = 0, moved_d2h = 0, moved_d2d = 0;   // bytes moved by the last budget change
    // budget change in progress
    int phase = kPhaseIdle;
    bool compact_wanted = false;
    std::deque<Move> todo;             // moves of the current phase that have not been issued
    std::deque<MoveBatch> inflight;    // issued, copy not yet known to have landed
    std::deque<Limbo> limbo;           // landed and switched over, old places not yet released
    std::vector<int32_t> to_load;      // lists to bring into HBM once evictions and compaction are over
    std::vector<char> seg_skip;        // HBM segments that compaction could not empty
    size_t inflight_bytes = 0;
    int64_t pending_lists = 0, pending_bytes = 0;   // lists that still have to change tier
    int move_rc = 0;                   // why the last change stopped early (0: it did not)
    std::string move_msg;
    hipStream_t move_stream = nullptr, patch_stream = nullptr;
    hipEvent_t ev_search_end = nullptr;   // = sc[0].end: searches on one stream (the only kind while lists move) use set 0
    bool search_end_recorded = false;
    std::vector<hipEvent_t> spare_events;
    std::vector<const void**> spare_tables;
    const void** h_list_ptr = nullptr; // pinned host mirror of d_list_ptr
    // streaming of host-resident lists
    hipStream_t side[kMaxSide] = {};   // copy streams for host-resident lists (chunks alternate)
    char* stage[kMaxStage] = {};
    hipEvent_t stage_ready[kMaxStage][kMaxSide] = {}, stage_free[kMaxStage] = {};
    bool stage_used[kMaxStage] = {};
    size_t stage_bytes = 0;
    int nstage = 0;
    hipEvent_t ev_probes = nullptr, ev_done = nullptr;
    bool done_recorded = false;
    // search state
    Scratch sc[kSets];                 // queued searches go round the sets; searches on one stream use set 0
    Scratch sc_static;                 // slices of the per-device static array (ivf_search_noalloc)
    char* static_base = nullptr;       // device address of that array on this index's device
    Scratch* last_sc = nullptr;        // set of the last search (introspection calls read it)
    unsigned long long* h_counters = nullptr;   // pinned landing place of a set's counters
    int prune_blocks = 0, prune_j = 0;   // bound kept by the scan for the current search (see k_scan)
    int last_nq = 0, last_nprobe = 0;
    hipStream_t last_stream = nullptr;
    bool last_offload = false;
    // queued searches (ivf_search_queued): a search's front stages run on one of two
    // front streams (taken in turn: under a scan these latency-bound kernels run several
    // times slower than alone, and two searches' worth side by side keep up with the scans),
    // its scan on pipe_scan behind the scan before it, its final selection on the caller's stream
    hipStream_t pipe_front[2] = {}, pipe_scan = nullptr;
    // These three and the caller's stream should sit on four different hardware queues (a
    // process has four; streams that share one run one after the other, whatever their
    // events say).  Which queue a stream gets cannot be asked, so the first queued search
    // finds out by trial which streams run side by side (pick_pipe_streams).
    bool pipe_picked = false;
    int pipe_pick_tries = 0;
    hipStream_t pipe_caller = nullptr;  // the caller's stream that the three were picked against
    hipEvent_t ev_trial[2] = {};        // timing events of the trials
    uint64_t queued_count = 0;
    hipEvent_t ev_front[kSets] = {}, ev_scan[kSets] = {};
    int next_set = 0;
    bool last_queued = false;
    ivf_search_stats last_stats = {};
    int timing = 0;                    // 0 off, 1 every stage, 2 scan and streaming stages only
    hipEvent_t ev[kTimingSlots][kEvPerSearch] = {};
    bool ev_created = false;
    bool ev_queued[kTimingSlots] = {};  // the slot's search was a queued one: only its scan was timed
    int64_t timed_searches = 0;        // searches recorded since timing was switched on
    // options
    int64_t opt_queue_min_mb = 256, opt_queue_fronts = 0, opt_scan_split = 0, opt_scan_unroll = 16, opt_scan_waves = 4, opt_scan_prune = 1, opt_host_direct = 1, opt_nside = 4, opt_policy = 0, opt_segment_mb = 2048, opt_stage_mb = 64,
            opt_nstage = 3, opt_move_chunk_kb = 64 << 10, opt_move_inflight_kb = 4 << 20, opt_sel_threads = 0, opt_regroup_fused = 1;
};

