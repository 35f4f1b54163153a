// Host side of the IVF retrieval library: index storage, placement between HBM and
// pinned host memory, and the per-search launch sequence.  Exports the C ABI declared
// in include/ivf.h.
#include "ivf_host.h"
#include "ivf_moves.h"

#include <mutex>

// Scratch memory of ivf_search_noalloc: one array per GPU that loads the library, held
// until the process ends and shared by every index on that GPU.  In host code the name
// is only a handle for hipGetSymbolAddress; kernels get the address looked up there.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
struct StaticScratchDevice {
    char* base = nullptr;            // device address of `scratch` on this GPU
    hipEvent_t last_use = nullptr;   // behind the last search that used the array
    bool used = false;
};
StaticScratchDevice g_static[kMaxDevices];
std::mutex g_static_mu;

// Looks the array's address up once per device (the device must be current).
int static_scratch_init(int device) {
    if (device < 0 || device >= kMaxDevices) return fail(IVF_ERR_LIMIT, "HIP device %d: at most %d devices", device, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_static_mu);
    StaticScratchDevice& dv = g_static[device];
    if (dv.base) return 0;
    void* ptr = nullptr;
    HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return fail(IVF_ERR_HIP, "hipGetSymbolAddress gave no address for the static scratch array");
    HIP_TRY(hipEventCreateWithFlags(&dv.last_use, hipEventDisableTiming));
    dv.base = static_cast<char*>(ptr);
    return 0;
}

void free_scratch(Scratch& s) {
    const hipEvent_t end = s.end;                // the index's, not the buffers'
    if (s.carved) {                              // slices of a region that is not ours to free
        s = Scratch();
        s.end = end;
        return;
    }
    dfree(s.S); dfree(s.tmax); dfree(s.probes); dfree(s.zeroed); dfree(s.pair_start);
    dfree(s.sblk_start); dfree(s.item_start); dfree(s.wg_totals); dfree(s.pair_flat);
    dfree(s.pair_of_probe); dfree(s.items); dfree(s.stream_items);
    dfree(s.scores); dfree(s.bmax); dfree(s.pq_tables); dfree(s.q_stage);
    if (s.h_probes) (void)hipHostFree(s.h_probes);
    if (s.h_items) (void)hipHostFree(s.h_items);
    s = Scratch();
    s.end = end;
}

void free_staging(ivf_index* x) {
    for (int i = 0; i < kMaxStage; ++i) {
        if (x->stage[i]) (void)hipFree(x->stage[i]);
        x->stage[i] = nullptr;
        x->stage_used[i] = false;
    }
    x->nstage = 0;
    x->stage_bytes = 0;
}

void free_index_data(ivf_index* x) {
    dfree(x->d_centroids); dfree(x->d_offsets); dfree(x->d_len);
    dfree(x->d_nblk); dfree(x->d_list_ptr); dfree(x->d_ids_pos); dfree(x->d_id_sorted);
    dfree(x->d_rank_of_pos); dfree(x->d_hits);
    if (x->h_list_ptr) { (void)hipHostFree(x->h_list_ptr); x->h_list_ptr = nullptr; }
    moves_reset(x);
    pool_free_all(x->dpool);
    pool_free_all(x->hpool);
    free_staging(x);
    for (int p = 0; p < kSets; ++p) free_scratch(x->sc[p]);
    free_scratch(x->sc_static);
    x->last_sc = nullptr;
    x->last_nq = 0;
    x->ready = x->uploading = false;
    x->resident_lists = 0;
}

template <class T>
int dalloc(T*& p, size_t count, size_t& total) {
    dfree(p);
    size_t bytes = std::max<size_t>(count * sizeof(T), 256);
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&p), bytes);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        p = nullptr;
        return fail(IVF_ERR_OOM_DEVICE, "hipMalloc of %zu bytes failed: %s", bytes, hipGetErrorString(e));
    }
    total += bytes;
    return 0;
}

int64_t block_bound(const ivf_index* x, int64_t nq, int nprobe) {
    size_t p = std::min<size_t>((size_t)nprobe, x->top_nblk_prefix.size() - 1);
    return nq * x->top_nblk_prefix[p];
}

int ensure_scratch(ivf_index* x, Scratch& s, int64_t nq, int nprobe, bool offload, bool q_host) {
    const int64_t ntile = (x->nlist + kCoarseTile - 1) / kCoarseTile;
    const size_t npairs = (size_t)nq * nprobe;
    const size_t nblocks = (size_t)std::max<int64_t>(1, block_bound(x, nq, nprobe));
    int rc;
    if ((size_t)nq * x->nlist > s.cap_q_nlist) {
        if ((rc = dalloc(s.S, (size_t)nq * x->nlist, s.bytes))) return rc;
        s.cap_q_nlist = (size_t)nq * x->nlist;
    }
    if ((size_t)nq * ntile > s.cap_q_ntile) {
        if ((rc = dalloc(s.tmax, (size_t)nq * ntile, s.bytes))) return rc;
        s.cap_q_ntile = (size_t)nq * ntile;
    }
    if (x->nlist > s.cap_nlist || (size_t)nq > s.cap_zero_q) {
        const size_t qcap = std::max<size_t>((size_t)nq, s.cap_zero_q);
        if ((rc = dalloc(s.zeroed, 2 * (size_t)x->nlist + 16 + 2 * kNumCounters + 2 * qcap, s.bytes))) return rc;
        s.counters = reinterpret_cast<unsigned long long*>(s.zeroed + 2 * (size_t)x->nlist + 16);
        s.qthr = s.counters + kNumCounters;
        s.cap_zero_q = qcap;
    }
    if (x->nlist > s.cap_nlist) {
        if ((rc = dalloc(s.wg_totals, kScanVals * (((size_t)x->nlist + kScanThreadsShared - 1) / kScanThreadsShared), s.bytes))) return rc;
        if ((rc = dalloc(s.pair_start, (size_t)x->nlist, s.bytes))) return rc;
        if ((rc = dalloc(s.sblk_start, (size_t)x->nlist, s.bytes))) return rc;
        if ((rc = dalloc(s.item_start, (size_t)x->nlist, s.bytes))) return rc;
        s.cap_nlist = x->nlist;
    }
    if (npairs > s.cap_pairs) {
        if ((rc = dalloc(s.probes, npairs, s.bytes))) return rc;
        if ((rc = dalloc(s.pair_flat, npairs, s.bytes))) return rc;
        if ((rc = dalloc(s.pair_of_probe, npairs, s.bytes))) return rc;
        s.cap_pairs = npairs;
    }
    if (nblocks > s.cap_blocks) {
        if ((rc = dalloc(s.items, nblocks, s.bytes))) return rc;
        if ((rc = dalloc(s.scores, nblocks * kLanes, s.bytes))) return rc;
        if ((rc = dalloc(s.bmax, nblocks, s.bytes))) return rc;
        s.cap_blocks = nblocks;
    }
    if (x->dtype == IVF_PQ8 && (size_t)nq > s.cap_pq_q) {
        if ((rc = dalloc(s.pq_tables, (size_t)nq * x->pq_m * 256, s.bytes))) return rc;
        s.cap_pq_q = (size_t)nq;
    }
    if (q_host && (size_t)nq * x->d > s.cap_q_stage) {
        if ((rc = dalloc(s.q_stage, (size_t)nq * x->d, s.bytes))) return rc;
        s.cap_q_stage = (size_t)nq * x->d;
    }
    if (offload) {
        if (nblocks > s.cap_stream_items) {
            if ((rc = dalloc(s.stream_items, nblocks, s.bytes))) return rc;
            s.cap_stream_items = nblocks;
        }
        if (npairs > s.h_probes_cap) {
            if (s.h_probes) (void)hipHostFree(s.h_probes);
            s.h_probes = nullptr;
            if (hipHostMalloc(reinterpret_cast<void**>(&s.h_probes), npairs * sizeof(int32_t)) != hipSuccess) {
                (void)hipGetLastError();
                return fail(IVF_ERR_OOM_HOST, "pinned allocation of the probe mirror failed");
            }
            s.h_probes_cap = npairs;
        }
        if (nblocks > s.h_items_cap) {
            if (s.h_items) (void)hipHostFree(s.h_items);
            s.h_items = nullptr;
            if (hipHostMalloc(reinterpret_cast<void**>(&s.h_items), nblocks * sizeof(ScanItem)) != hipSuccess) {
                (void)hipGetLastError();
                return fail(IVF_ERR_OOM_HOST, "pinned allocation of the item mirror failed");
            }
            s.h_items_cap = nblocks;
        }
    }
    return 0;
}

// The same buffers as slices of one region that the caller owns (256-byte aligned, in a
// fixed order).  Returns the bytes the search needs; `s` is filled only if they fit in `cap`.
size_t carve_scratch(const ivf_index* x, int64_t nq, int nprobe, bool q_host, char* base, size_t cap, Scratch& s) {
    const size_t nlist = (size_t)x->nlist;
    const size_t ntile = (nlist + kCoarseTile - 1) / kCoarseTile;
    const size_t npairs = (size_t)nq * nprobe;
    const size_t nblocks = (size_t)std::max<int64_t>(1, block_bound(x, nq, nprobe));
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t o = off;
        off += (std::max<size_t>(bytes, 256) + 255) & ~(size_t)255;
        return o;
    };
    const size_t o_S = take(4 * (size_t)nq * nlist), o_tmax = take(4 * (size_t)nq * ntile);
    const size_t o_zero = take(4 * (2 * nlist + 16 + 2 * kNumCounters + 2 * (size_t)nq));
    const size_t o_wg = take(4 * kScanVals * ((nlist + kScanThreadsShared - 1) / kScanThreadsShared));
    const size_t o_ps = take(4 * nlist), o_sb = take(4 * nlist), o_is = take(4 * nlist);
    const size_t o_pr = take(4 * npairs), o_pf = take(4 * npairs), o_pp = take(4 * npairs);
    const size_t o_it = take(sizeof(ScanItem) * nblocks), o_sc = take(4 * nblocks * kLanes), o_bm = take(4 * nblocks);
    const size_t o_pq = x->dtype == IVF_PQ8 ? take(4 * (size_t)nq * x->pq_m * 256) : 0;
    const size_t o_qs = q_host ? take(4 * (size_t)nq * x->d) : 0;
    if (off > cap) return off;
    const hipEvent_t end = s.end;
    const bool end_recorded = s.end_recorded;
    s = Scratch();
    s.end = end;
    s.end_recorded = end_recorded;
    s.carved = true;
    s.S = reinterpret_cast<float*>(base + o_S);
    s.tmax = reinterpret_cast<float*>(base + o_tmax);
    s.zeroed = reinterpret_cast<int*>(base + o_zero);
    s.counters = reinterpret_cast<unsigned long long*>(s.zeroed + 2 * nlist + 16);
    s.qthr = s.counters + kNumCounters;
    s.wg_totals = reinterpret_cast<uint32_t*>(base + o_wg);
    s.pair_start = reinterpret_cast<uint32_t*>(base + o_ps);
    s.sblk_start = reinterpret_cast<uint32_t*>(base + o_sb);
    s.item_start = reinterpret_cast<uint32_t*>(base + o_is);
    s.probes = reinterpret_cast<int32_t*>(base + o_pr);
    s.pair_flat = reinterpret_cast<uint32_t*>(base + o_pf);
    s.pair_of_probe = reinterpret_cast<uint32_t*>(base + o_pp);
    s.items = reinterpret_cast<ScanItem*>(base + o_it);
    s.scores = reinterpret_cast<float*>(base + o_sc);
    s.bmax = reinterpret_cast<float*>(base + o_bm);
    if (x->dtype == IVF_PQ8) s.pq_tables = reinterpret_cast<float*>(base + o_pq);
    if (q_host) s.q_stage = reinterpret_cast<float*>(base + o_qs);
    s.bytes = off;
    return off;
}

// One search as the launch sequence sees it.
struct SearchCtx {
    const float* Q = nullptr;
    bool q_host = false;               // Q is pinned host memory: the search starts with a copy to the device
    int64_t nq = 0;
    int nprobe = 0, k = 0;
    int64_t* out_ids = nullptr;
    float* out_scores = nullptr;
    int nlist = 0, ntile = 0, npairs = 0;
    bool offload = false;              // host-resident lists are copied to staging buffers
    bool moving = false;               // a budget change was under way when the search was issued
    int prune_blocks = 0, prune_j = 0; // bound kept by the scan (see k_scan)
    // Events tied to the scan kernel's own start and end (either may be null).  Bound to the
    // dispatch itself, they cost no packet of their own on the stream, unlike a recorded
    // event, and read the kernel's duration without the launch gap around it.
    hipEvent_t scan_start = nullptr, scan_stop = nullptr;
};

template <int ST, int U, int WAVES>
void launch_scan_k(ivf_index* x, Scratch& s, const SearchCtx& c, size_t work_items, hipStream_t st, const ScanItem* items,
                   const unsigned long long* n_dev, uint32_t n_host, const float* Q) {
    const dim3 grid((unsigned)((work_items + WAVES - 1) / WAVES));
    hipExtLaunchKernelGGL((k_scan<ST, U, WAVES>), grid, dim3(WAVES * 64), 0, st, c.scan_start, c.scan_stop, 0, items, n_dev,
                          n_host, Q, x->d, s.scores, s.bmax, s.qthr, c.prune_blocks, c.prune_j);
}

template <int ST, int U>
void launch_scan_w(ivf_index* x, Scratch& s, const SearchCtx& c, size_t work_items, hipStream_t st, const ScanItem* items,
                   const unsigned long long* n_dev, uint32_t n_host, const float* Q) {
    switch ((int)x->opt_scan_waves) {
        case 1: launch_scan_k<ST, U, 1>(x, s, c, work_items, st, items, n_dev, n_host, Q); break;
        case 2: launch_scan_k<ST, U, 2>(x, s, c, work_items, st, items, n_dev, n_host, Q); break;
        case 8: launch_scan_k<ST, U, 8>(x, s, c, work_items, st, items, n_dev, n_host, Q); break;
        default: launch_scan_k<ST, U, 4>(x, s, c, work_items, st, items, n_dev, n_host, Q);
    }
}

// Wavefronts that share one block.  By default a wavefront's share is kept at 48 KiB or
// more (shorter shares lose to the fixed cost per item): a function of the stored vector's
// size alone, so that an index always adds its partial sums in the same order.
int scan_split_of(const ivf_index* x) {
    if (x->opt_scan_split) return (int)x->opt_scan_split;
    const size_t share = (size_t)48 << 10;
    return x->block_bytes >= 4 * share ? 4 : x->block_bytes >= 2 * share ? 2 : 1;
}

template <int ST, int SPLIT>
void launch_scan_split(ivf_index* x, Scratch& s, const SearchCtx& c, size_t work_items, hipStream_t st, const ScanItem* items,
                       const unsigned long long* n_dev, uint32_t n_host, const float* Q) {
    constexpr int per_wg = 4 / SPLIT;                        // items per workgroup of four wavefronts
    const dim3 grid((unsigned)((work_items + per_wg - 1) / per_wg));
    const int chunks = x->d / Store<ST>::E / SPLIT;          // per wavefront (the shorter share if uneven)
    // the widest register buffers that the share of a wavefront fills without a remainder
    if (chunks % 16 == 0 && x->opt_scan_unroll == 16)
        hipExtLaunchKernelGGL((k_scan_split<ST, 16, SPLIT>), grid, dim3(256), 0, st, c.scan_start, c.scan_stop, 0, items, n_dev,
                              n_host, Q, x->d, s.scores, s.bmax, s.qthr, c.prune_blocks, c.prune_j);
    else
        hipExtLaunchKernelGGL((k_scan_split<ST, 8, SPLIT>), grid, dim3(256), 0, st, c.scan_start, c.scan_stop, 0, items, n_dev,
                              n_host, Q, x->d, s.scores, s.bmax, s.qthr, c.prune_blocks, c.prune_j);
}

template <int ST>
void launch_scan_split_s(ivf_index* x, Scratch& s, const SearchCtx& c, size_t work_items, hipStream_t st, const ScanItem* items,
                         const unsigned long long* n_dev, uint32_t n_host, const float* Q) {
    if (scan_split_of(x) == 2) launch_scan_split<ST, 2>(x, s, c, work_items, st, items, n_dev, n_host, Q);
    else launch_scan_split<ST, 4>(x, s, c, work_items, st, items, n_dev, n_host, Q);
}

// work_items: number of items (an upper bound is enough, excess wavefronts exit)
void launch_scan(ivf_index* x, Scratch& s, const SearchCtx& c, size_t work_items, hipStream_t st, const ScanItem* items,
                 const unsigned long long* n_dev, uint32_t n_host, const float* Q) {
    const int U = (int)x->opt_scan_unroll;
    if (scan_split_of(x) > 1) {                    // several wavefronts per item
        if (x->dtype == IVF_FP16) launch_scan_split_s<kF16>(x, s, c, work_items, st, items, n_dev, n_host, Q);
        else if (x->dtype == IVF_INT8) launch_scan_split_s<kI8>(x, s, c, work_items, st, items, n_dev, n_host, Q);
        else launch_scan_split_s<kF32>(x, s, c, work_items, st, items, n_dev, n_host, Q);
        return;
    }
    if (x->dtype == IVF_FP16) {
        if (U == 8) launch_scan_w<kF16, 8>(x, s, c, work_items, st, items, n_dev, n_host, Q);
        else launch_scan_w<kF16, 16>(x, s, c, work_items, st, items, n_dev, n_host, Q);
    } else if (x->dtype == IVF_INT8) {
        if (U == 8) launch_scan_w<kI8, 8>(x, s, c, work_items, st, items, n_dev, n_host, Q);
        else launch_scan_w<kI8, 16>(x, s, c, work_items, st, items, n_dev, n_host, Q);
    } else {
        if (U == 8) launch_scan_w<kF32, 8>(x, s, c, work_items, st, items, n_dev, n_host, Q);
        else launch_scan_w<kF32, 16>(x, s, c, work_items, st, items, n_dev, n_host, Q);
    }
}

int ensure_staging(ivf_index* x) {
    size_t max_list_bytes = 0;
    for (int64_t l = 0; l < x->nlist; ++l)
        max_list_bytes = std::max(max_list_bytes, (size_t)x->nblk[l] * x->block_bytes);
    size_t want = std::max<size_t>((size_t)x->opt_stage_mb << 20, max_list_bytes);
    int nst = (int)std::min<int64_t>(kMaxStage, std::max<int64_t>(2, x->opt_nstage));
    if (x->nstage == nst && x->stage_bytes >= want) return 0;
    free_staging(x);
    for (int i = 0; i < nst; ++i) {
        hipError_t e = hipMalloc(reinterpret_cast<void**>(&x->stage[i]), want);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            free_staging(x);
            return fail(IVF_ERR_OOM_DEVICE, "staging buffer of %zu bytes: %s", want, hipGetErrorString(e));
        }
    }
    x->nstage = nst;
    x->stage_bytes = want;
    return 0;
}

// The host-resident part of a search: mirror the device's pair numbering, pack the
// probed host lists into staging-sized chunks, copy each chunk on the side stream and
// scan it on the caller's stream as soon as it has landed.
int stream_host_lists(ivf_index* x, Scratch& s, const SearchCtx& c, hipStream_t st) {
    const float* Q = c.Q;
    const int64_t nq = c.nq;
    const int nprobe = c.nprobe;
    HIP_TRY(hipEventSynchronize(x->ev_probes));
    const int nside = (int)std::min<int64_t>(kMaxSide, std::max<int64_t>(1, x->opt_nside));
    for (int i = 0; i < kMaxSide; ++i) {
        int rc = need_stream(x->side[i]);
        if (rc) return rc;
    }
    for (int i = 0; i < kMaxSide; ++i) HIP_TRY(hipStreamSynchronize(x->side[i]));   // pinned item mirror of the previous search is free
    const size_t npairs = (size_t)nq * nprobe;
    std::vector<std::pair<int32_t, uint32_t>> pl(npairs);
    for (size_t f = 0; f < npairs; ++f) pl[f] = {s.h_probes[f], (uint32_t)f};
    std::sort(pl.begin(), pl.end());
    ivf_search_stats& stt = x->last_stats;
    stt = ivf_search_stats();
    stt.pairs = (int64_t)npairs;

    struct HostList { int32_t l; uint32_t cnt, ps, sb; size_t first; };   // first: index into pl
    std::vector<HostList> hl;
    uint32_t ps = 0, sb = 0;
    for (size_t i = 0; i < npairs;) {
        size_t j = i;
        while (j < npairs && pl[j].first == pl[i].first) ++j;
        int32_t l = pl[i].first;
        uint32_t cnt = (uint32_t)(j - i);
        stt.unique_lists += 1;
        stt.scanned_vectors += x->len[l];
        int64_t bytes = (int64_t)x->len[l] * (int64_t)x->row_bytes;
        stt.scan_bytes += bytes;
        if (x->dev_ptr[l]) {
            stt.scan_bytes_resident += bytes;
            stt.scan_items += (int64_t)x->nblk[l] * ((cnt + kQB - 1) / kQB);
        } else {
            stt.scan_bytes_streamed += bytes;
            if (x->nblk[l] > 0) hl.push_back({l, cnt, ps, sb, i});
        }
        ps += cnt;
        sb += cnt * (uint32_t)x->nblk[l];
        i = j;
    }
    if (x->done_recorded)
        for (int i = 0; i < nside; ++i) HIP_TRY(hipStreamWaitEvent(x->side[i], x->ev_done, 0));

    size_t item_off = 0;
    size_t i = 0;
    int chunk = 0;
    while (i < hl.size()) {
        const int slot = chunk % x->nstage;
        size_t used = 0, j = i;
        while (j < hl.size()) {
            size_t b = (size_t)x->nblk[hl[j].l] * x->block_bytes;
            if (used + b > x->stage_bytes) break;
            used += b;
            ++j;
        }
        if (j == i) return fail(IVF_ERR_LIMIT, "staging buffer smaller than a list");
        // The copies of a chunk go round the copy streams: a copy of one list (~2 MB) is too
        // short to reach the link's rate by itself, two or three of them side by side do.
        if (x->stage_used[slot])
            for (int sd = 0; sd < nside; ++sd) HIP_TRY(hipStreamWaitEvent(x->side[sd], x->stage_free[slot], 0));
        // copies: merge lists that are neighbours in the host arena
        size_t dst_off = 0;
        size_t a = i;
        const size_t item_begin = item_off;
        int ncopy = 0;
        while (a < j) {
            hipStream_t side = x->side[ncopy % nside];
            ++ncopy;
            const char* src = x->host_ptr[hl[a].l];
            size_t bytes = (size_t)x->nblk[hl[a].l] * x->block_bytes;
            size_t e = a + 1;
            while (e < j && x->host_ptr[hl[e].l] == src + bytes) {
                bytes += (size_t)x->nblk[hl[e].l] * x->block_bytes;
                ++e;
            }
            HIP_TRY(hipMemcpyAsync(x->stage[slot] + dst_off, src, bytes, hipMemcpyHostToDevice, side));
            dst_off += bytes;
            a = e;
        }
        // items of the chunk
        size_t loff = 0;
        for (size_t t = i; t < j; ++t) {
            const HostList& h = hl[t];
            const uint32_t nb = (uint32_t)x->nblk[h.l];
            const uint32_t groups = (h.cnt + kQB - 1) / kQB;
            for (uint32_t g = 0; g < groups; ++g)
                for (uint32_t b = 0; b < nb; ++b) {
                    ScanItem it;
                    it.data = x->stage[slot] + loff + (size_t)b * x->block_bytes;
                    it.sblk = h.sb + g * kQB * nb + b;
                    it.nblk = nb;
                    const uint32_t nqg = std::min<uint32_t>(kQB, h.cnt - g * kQB);
                    for (uint32_t jq = 0; jq < (uint32_t)kQB; ++jq)
                        it.q[jq] = (uint16_t)(pl[h.first + g * kQB + std::min(jq, nqg - 1)].second / (uint32_t)nprobe);
                    it.nq = (uint16_t)nqg;
                    it.nvalid = (uint16_t)std::min<uint32_t>(64u, (uint32_t)x->len[h.l] - b * 64u);
                    it.shared = groups > 1 ? 1u : 0u;
                    s.h_items[item_off + item_slot(g, b, groups)] = it;
                }
            item_off += (size_t)groups * nb;
            loff += (size_t)nb * x->block_bytes;
        }
        const size_t nitems = item_off - item_begin;
        HIP_TRY(hipMemcpyAsync(s.stream_items + item_begin, s.h_items + item_begin,
                               nitems * sizeof(ScanItem), hipMemcpyHostToDevice, x->side[ncopy % nside]));
        for (int sd = 0; sd < std::min(nside, ncopy + 1); ++sd) {
            HIP_TRY(hipEventRecord(x->stage_ready[slot][sd], x->side[sd]));
            HIP_TRY(hipStreamWaitEvent(st, x->stage_ready[slot][sd], 0));
        }
        launch_scan(x, s, c, nitems, st, s.stream_items + item_begin, nullptr, (uint32_t)nitems, Q);
        HIP_TRY(hipGetLastError());
        HIP_TRY(hipEventRecord(x->stage_free[slot], st));
        x->stage_used[slot] = true;
        stt.scan_items += (int64_t)nitems;
        i = j;
        ++chunk;
    }
    return 0;
}

int check_ready(const ivf_index* x) {
    if (!x) return fail(IVF_ERR_INVALID, "index is NULL");
    if (!x->ready) return fail(IVF_ERR_INVALID, "index has no uploaded data");
    return 0;
}

// Argument checks shared by the search entry points.  Returns a negative error, 1 if there
// is nothing to do (nq = 0), 0 otherwise with `c` filled in.
int search_args(ivf_index* x, const float* queries, int64_t nq, int nprobe, int k, int64_t* out_ids,
                float* out_scores, SearchCtx& c) {
    int rc = check_ready(x);
    if (rc) return rc;
    if (nq < 0) return fail(IVF_ERR_INVALID, "nq must be non-negative");
    if (nq == 0) return 1;
    if (!queries || !out_ids || !out_scores) return fail(IVF_ERR_INVALID, "queries, out_ids or out_scores is NULL");
    if (nprobe <= 0 || k <= 0) return fail(IVF_ERR_INVALID, "nprobe and k must be positive");
    if (k > kMaxK) return fail(IVF_ERR_LIMIT, "k above %d", kMaxK);
    if (nprobe > x->nlist) nprobe = (int)x->nlist;
    if (nprobe > kMaxK) return fail(IVF_ERR_LIMIT, "nprobe above %d", kMaxK);
    if (nq > 65535) return fail(IVF_ERR_LIMIT, "nq above 65535");
    if ((uint64_t)nq * (uint64_t)nprobe >= (1ull << 31)) return fail(IVF_ERR_LIMIT, "nq*nprobe above 2^31");
    if ((uint64_t)block_bound(x, nq, nprobe) >= (1ull << 31)) return fail(IVF_ERR_LIMIT, "batch too large for one call");
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != x->device)
        return fail(IVF_ERR_INVALID, "the index lives on HIP device %d but the current device is %d", x->device, dev);
    hipPointerAttribute_t qa;
    if (hipPointerGetAttributes(&qa, queries) != hipSuccess) {
        (void)hipGetLastError();
        return fail(IVF_ERR_INVALID, "queries is neither device memory nor pinned host memory (hipHostMalloc)");
    }
    if (qa.type != hipMemoryTypeHost && qa.type != hipMemoryTypeDevice && qa.type != hipMemoryTypeManaged &&
        qa.type != hipMemoryTypeUnified)
        return fail(IVF_ERR_INVALID, "queries is neither device memory nor pinned host memory (hipHostMalloc)");
    c.q_host = qa.type == hipMemoryTypeHost;
    c.Q = queries; c.nq = nq; c.nprobe = nprobe; c.k = k; c.out_ids = out_ids; c.out_scores = out_scores;
    c.nlist = (int)x->nlist;
    c.ntile = (c.nlist + kCoarseTile - 1) / kCoarseTile;
    c.npairs = (int)(nq * nprobe);
    c.offload = x->resident_lists < x->nlist && !x->opt_host_direct;
    if (x->dtype == IVF_PQ8 && c.offload)
        return fail(IVF_ERR_INVALID, "product-quantised lists in pinned host memory are read in place: "
                                     "the staged mode (host_direct = 0) does not take them");
    return 0;
}

// Searches share scratch memory: a search starts behind the event that the last user of
// its scratch set left behind its last kernel (no host wait; nothing at all when that
// event was recorded on the same stream).  The stream of an earlier search is never
// touched again: the caller may have destroyed it.  `first` is the stream of this search's
// first kernel, `st` the caller's.
bool stream_is_capturing(hipStream_t st) {
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cs) != hipSuccess) { (void)hipGetLastError(); return false; }
    return cs == hipStreamCaptureStatusActive;
}

int order_after_last_use(Scratch& s, hipStream_t st, hipStream_t first) {
    if (!s.end_recorded) return 0;
    if (stream_is_capturing(st)) return 0;            // a captured search is kernel launches only; its place among
                                                      // the other searches is where the caller launches the graph
    HIP_TRY(hipStreamWaitEvent(first, s.end, 0));
    return 0;
}

// What a search on one stream does before its first kernel.
int search_prologue(ivf_index* x, hipStream_t st, SearchCtx& c) {
    int rc;
    c.moving = moves_active(x);
    if (c.moving) {
        // a budget change is under way: take over what has landed, issue more copies, and
        // let this search start only behind the latest update of the address table
        if ((rc = moves_advance(x))) return rc;
        if (!x->limbo.empty()) HIP_TRY(hipStreamWaitEvent(st, x->limbo.back().after, 0));
    }
    c.offload = x->resident_lists < x->nlist && !x->opt_host_direct;
    if (x->dtype == IVF_PQ8 && c.offload)
        return fail(IVF_ERR_INVALID, "product-quantised lists in pinned host memory are read in place: "
                                     "the staged mode (host_direct = 0) does not take them");
    if (c.offload && (rc = ensure_staging(x))) return rc;
    return 0;
}

// Running lower bound of each query's k-th best score, kept by the scan so that it can
// skip storing blocks that cannot matter: from one block's k-th largest value (k <= 64) or
// from the two best blocks' ceil(k/2)-th largest (k <= 128).  Small plans run as one wave
// of work items, where nothing has a bound to prune by yet.
void search_set_pruning(const ivf_index* x, SearchCtx& c) {
    const bool small_plan = x->opt_scan_prune != 2 && block_bound(x, c.nq, c.nprobe) < 32768;
    // Over product-quantisation codes a wavefront scans block after block, and the bound
    // costs it more at every block (half as much again at 100 M vectors) than the stores
    // it saves: no pruning there unless asked for ("scan_prune" = 2).
    const bool pq_default = x->dtype == IVF_PQ8 && x->opt_scan_prune != 2;
    if (!x->opt_scan_prune || c.k > 128 || small_plan || pq_default) { c.prune_blocks = 0; c.prune_j = 0; }
    else if (c.k <= 64) { c.prune_blocks = 1; c.prune_j = c.k; }
    else { c.prune_blocks = 2; c.prune_j = (c.k + 1) / 2; }
}

void enqueue_coarse(ivf_index* x, Scratch& s, const SearchCtx& c, hipStream_t st) {
    const int nz = (int)(2 * (size_t)c.nlist + 16 + 2 * kNumCounters + 2 * (size_t)c.nq);   // cleared by the coarse kernel
    // Query rows per wavefront: as many as possible (each centroid row is then fetched
    // once), but few enough that the grid still offers every SIMD a wavefront.
    dim3 grid((unsigned)((c.nlist + kCoarseNT - 1) / kCoarseNT), 1);
    const int64_t simds = (int64_t)x->cus * 4, waves_x = (int64_t)grid.x * 4;
    const int64_t nq = c.nq;
    int mt = nq > 64 ? 4 : nq > 32 ? 2 : 1;
    while (mt > 1 && waves_x * ((nq + 32 * mt - 1) / (32 * mt)) < simds) mt >>= 1;
    grid.y = (unsigned)((nq + 32 * mt - 1) / (32 * mt));
    if (mt == 1)
        hipLaunchKernelGGL((k_coarse<1>), grid, dim3(256), 0, st, c.Q, x->d_centroids, s.S, s.tmax, (int)nq, c.nlist, x->d, c.ntile, s.zeroed, nz);
    else if (mt == 2)
        hipLaunchKernelGGL((k_coarse<2>), grid, dim3(256), 0, st, c.Q, x->d_centroids, s.S, s.tmax, (int)nq, c.nlist, x->d, c.ntile, s.zeroed, nz);
    else
        hipLaunchKernelGGL((k_coarse<4>), grid, dim3(256), 0, st, c.Q, x->d_centroids, s.S, s.tmax, (int)nq, c.nlist, x->d, c.ntile, s.zeroed, nz);
}

// The selection kernels are chains of barriers and dependent loads: with little to select
// from, a workgroup of 4 wavefronts gets through them faster than one of 16.
void enqueue_probe_select(ivf_index* x, Scratch& s, const SearchCtx& c, hipStream_t st, bool under_a_scan) {
    int* hist = s.zeroed;
    // (under another search's scan only a workgroup of four wavefronts finds room on a compute unit)
    const bool small_probe = x->opt_sel_threads ? x->opt_sel_threads == 256 : (under_a_scan || c.ntile <= 128);
    if (small_probe)
        hipLaunchKernelGGL((k_probe_select<256>), dim3((unsigned)c.nq), dim3(256), 0, st, s.S, s.tmax, c.nlist, c.ntile, c.nprobe,
                           s.probes, hist);
    else
        hipLaunchKernelGGL((k_probe_select<kSelThreads>), dim3((unsigned)c.nq), dim3(kSelThreads), 0, st, s.S, s.tmax, c.nlist,
                           c.ntile, c.nprobe, s.probes, hist);
}

void enqueue_regroup(ivf_index* x, Scratch& s, const SearchCtx& c, hipStream_t st, bool under_a_scan) {
    int* hist = s.zeroed;
    int* cursor = s.zeroed + c.nlist;
    const int nlist = c.nlist, npairs = c.npairs, nprobe = c.nprobe;
    // One launch instead of four pays up to 1024 lists when the kernels have the GPU to
    // themselves.  Under the scan of another search every launch waits tens of
    // microseconds for room on a compute unit, so the single workgroup wins up to four
    // times that size.
    const int fuse = under_a_scan ? 4 : 1;
    if (x->opt_regroup_fused && nlist <= fuse * kFusedMaxLists && npairs <= fuse * kFusedMaxPairs) {
        // few lists and pairs: one workgroup does the whole regrouping in one launch (sixteen
        // wavefronts also under a scan: with four, each thread's share of the lists is a chain
        // of loads four times as long, and under a scan every link of it is slow — 250 us
        // against 110 at 4096 lists)
        hipLaunchKernelGGL((k_regroup_small<kScanThreads>), dim3(1), dim3(kScanThreads), 0, st, hist, x->d_nblk, x->d_len,
                           x->d_list_ptr, nlist, nprobe, x->block_bytes, s.probes, npairs, cursor, s.pair_start,
                           s.sblk_start, s.item_start, s.pair_flat, s.pair_of_probe, s.items, x->d_hits, s.counters);
    } else {
        if (under_a_scan) {
            constexpr int T = kScanThreadsShared;
            const unsigned wgs = (unsigned)((nlist + T - 1) / T);
            hipLaunchKernelGGL((k_list_partial<T>), dim3(wgs), dim3(T), 0, st, hist, x->d_nblk, x->d_len, x->d_list_ptr,
                               nlist, s.pair_start, s.sblk_start, s.item_start, s.wg_totals, s.counters);
            hipLaunchKernelGGL((k_list_finish<T>), dim3(wgs), dim3(T), 0, st, hist, nlist, (int)wgs, s.wg_totals,
                               s.pair_start, s.sblk_start, s.item_start);
        } else {
            constexpr int T = kScanThreads;
            const unsigned wgs = (unsigned)((nlist + T - 1) / T);
            hipLaunchKernelGGL((k_list_partial<T>), dim3(wgs), dim3(T), 0, st, hist, x->d_nblk, x->d_len, x->d_list_ptr,
                               nlist, s.pair_start, s.sblk_start, s.item_start, s.wg_totals, s.counters);
            hipLaunchKernelGGL((k_list_finish<T>), dim3(wgs), dim3(T), 0, st, hist, nlist, (int)wgs, s.wg_totals,
                               s.pair_start, s.sblk_start, s.item_start);
        }
        hipLaunchKernelGGL(k_pair_fill, dim3((unsigned)((npairs + 255) / 256)), dim3(256), 0, st, s.probes, npairs,
                           s.pair_start, cursor, s.pair_flat);
        hipLaunchKernelGGL(k_plan, dim3((unsigned)((nlist + 255) / 256)), dim3(256), 0, st, hist, x->d_nblk, x->d_len,
                           x->d_list_ptr, nlist, nprobe, x->block_bytes, s.pair_start, s.sblk_start, s.item_start,
                           s.pair_flat, s.pair_of_probe, s.items, x->d_hits);
    }
}

// The scan of every list the kernel can read (HBM-resident, or pinned host memory read in place).
void enqueue_scan_kernels(ivf_index* x, Scratch& s, const SearchCtx& c, hipStream_t st);

// c.scan_start / c.scan_stop, if set, end up around the scan: bound to the kernel where one
// kernel does the scan, recorded on the stream otherwise.
void enqueue_scan(ivf_index* x, Scratch& s, const SearchCtx& c, hipStream_t st) {
    const bool one_kernel = x->dtype != IVF_PQ8 && (x->resident_lists > 0 || x->opt_host_direct);
    if (!one_kernel && c.scan_start) (void)hipEventRecord(c.scan_start, st);
    enqueue_scan_kernels(x, s, c, st);
    if (!one_kernel && c.scan_stop) (void)hipEventRecord(c.scan_stop, st);
}

void enqueue_scan_kernels(ivf_index* x, Scratch& s, const SearchCtx& c, hipStream_t st) {
    if (x->dtype == IVF_PQ8) {
        // product-quantised lists: the queries' tables against the codebooks, then workgroups
        // that hold one query's table in LDS and scan a share of its probed lists: enough
        // shares for about four workgroups per compute unit, at most kPqWgLists lists each
        hipLaunchKernelGGL(k_pq_tables, dim3((unsigned)x->pq_m, (unsigned)c.nq), dim3(256), 0, st, c.Q, x->d_codebooks,
                           s.pq_tables, x->d, x->pq_m);
        const int64_t fewest = (c.nprobe + kPqWgLists - 1) / kPqWgLists;
        const int64_t parts = std::min<int64_t>(c.nprobe, std::max<int64_t>(fewest, (1024 + c.nq - 1) / c.nq));
        hipLaunchKernelGGL(k_pq_scan, dim3((unsigned)parts, (unsigned)c.nq), dim3(kPqThreads), (size_t)x->pq_m * 1024, st,
                           s.probes, s.pair_of_probe, s.pair_start, s.sblk_start, x->d_nblk, x->d_len, x->d_list_ptr, c.nprobe,
                           x->pq_m, s.pq_tables, s.scores, s.bmax, s.qthr, c.prune_blocks, c.prune_j);
        return;
    }
    if (x->resident_lists > 0 || x->opt_host_direct) {
        const int64_t bound = std::max<int64_t>(1, block_bound(x, c.nq, c.nprobe));
        launch_scan(x, s, c, (size_t)bound, st, s.items, s.counters + kCntItems, 0, c.Q);
    }
}

void enqueue_final_select(ivf_index* x, Scratch& s, const SearchCtx& c, hipStream_t st, bool under_a_scan) {
    const bool small_final = x->opt_sel_threads ? x->opt_sel_threads == 256 : (under_a_scan || block_bound(x, 1, c.nprobe) <= 128);
    ListTable lt{x->d_len, x->d_nblk, x->d_offsets};
    if (small_final)
        hipLaunchKernelGGL((k_final_select<256>), dim3((unsigned)c.nq), dim3(256), 0, st, s.probes, s.pair_of_probe,
                           s.pair_start, s.sblk_start, lt, s.bmax, s.scores, x->d_rank_of_pos, x->d_id_sorted, c.nprobe, c.k,
                           c.prune_blocks ? s.qthr : nullptr, c.out_ids, c.out_scores);
    else
        hipLaunchKernelGGL((k_final_select<kSelThreads>), dim3((unsigned)c.nq), dim3(kSelThreads), 0, st, s.probes,
                           s.pair_of_probe, s.pair_start, s.sblk_start, lt, s.bmax, s.scores, x->d_rank_of_pos,
                           x->d_id_sorted, c.nprobe, c.k, c.prune_blocks ? s.qthr : nullptr, c.out_ids, c.out_scores);
}

void search_epilogue(ivf_index* x, Scratch& s, const SearchCtx& c, hipStream_t st, bool queued) {
    x->last_sc = &s;
    x->last_nq = (int)c.nq;
    x->last_nprobe = c.nprobe;
    x->last_stream = st;
    x->last_offload = c.offload;
    x->last_queued = queued;
}

// The whole search as one chain of kernels on the caller's stream.
// Queries in pinned host memory: every kernel reads the copy that this puts in front of the
// search, on the stream of its first kernel (no stream or event of the caller's involved).
int stage_queries(ivf_index* x, Scratch& s, SearchCtx& c, hipStream_t first) {
    if (!c.q_host) return 0;
    HIP_TRY(hipMemcpyAsync(s.q_stage, c.Q, sizeof(float) * (size_t)c.nq * x->d, hipMemcpyHostToDevice, first));
    c.Q = s.q_stage;
    return 0;
}

int search_serial(ivf_index* x, Scratch& s, SearchCtx& c, hipStream_t st) {
    int rc;
    if ((rc = stage_queries(x, s, c, st))) return rc;
    search_set_pruning(x, c);
    const int tm = x->timing;                  // 0 off, 1 every stage, 2 the scan and streaming stages only
    hipEvent_t* evs = x->ev[x->timed_searches % kTimingSlots];
    int evi = 0;
    auto mark = [&]() {
        if (tm == 1 || (tm == 2 && evi >= 3 && evi <= 5)) (void)hipEventRecord(evs[evi], st);
        ++evi;
    };
    mark();   // 0
    enqueue_coarse(x, s, c, st);
    mark();   // 1
    enqueue_probe_select(x, s, c, st, false);
    mark();   // 2
    if (c.offload) {
        HIP_TRY(hipMemcpyAsync(s.h_probes, s.probes, sizeof(int32_t) * (size_t)c.npairs, hipMemcpyDeviceToHost, st));
        HIP_TRY(hipEventRecord(x->ev_probes, st));
    }
    enqueue_regroup(x, s, c, st, false);
    if (tm) { c.scan_start = evs[3]; c.scan_stop = evs[4]; }     // events 3 and 4 sit on the scan itself
    evi += 2;
    enqueue_scan(x, s, c, st);
    c.scan_start = c.scan_stop = nullptr;
    HIP_TRY(hipGetLastError());
    if (c.offload) {
        if ((rc = stream_host_lists(x, s, c, st))) return rc;
    }
    mark();   // 5
    enqueue_final_select(x, s, c, st, false);
    mark();   // 6
    HIP_TRY(hipGetLastError());
    if (c.offload) {
        HIP_TRY(hipEventRecord(x->ev_done, st));
        x->done_recorded = true;
    }
    // behind the last kernel: the next search on another stream starts after it, and old
    // places of moved lists are released only behind the searches that may read them
    // (not under stream capture: the captured search stays a chain of kernels)
    const bool moving = c.moving || moves_active(x);
    if (moving || !stream_is_capturing(st)) {
        HIP_TRY(hipEventRecord(s.end, st));
        s.end_recorded = true;
        if (moving) x->search_end_recorded = true;      // s is set 0 then, whose event is ev_search_end
    }
    search_epilogue(x, s, c, st, false);
    if (tm) {
        x->ev_queued[x->timed_searches % kTimingSlots] = false;
        x->timed_searches += 1;
    }
    return 0;
}


}  // namespace

extern "C" {

const char* ivf_last_error(void) { return g_err.c_str(); }

int ivf_index_create(ivf_index** out) {
    if (!out) return fail(IVF_ERR_INVALID, "out is NULL");
    *out = nullptr;
    ivf_index* x = new (std::nothrow) ivf_index();
    if (!x) return fail(IVF_ERR_OOM_HOST, "out of host memory");
    hipError_t e = hipGetDevice(&x->device);
    hipDeviceProp_t prop;
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, x->device);
    // The library's own streams are made when first needed (need_stream): a process has
    // four hardware queues, streams that share one run one after the other, and which
    // streams share depends on how many exist.
    for (int i = 0; e == hipSuccess && i < kSets; ++i) {
        e = hipEventCreateWithFlags(&x->ev_front[i], hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&x->ev_scan[i], hipEventDisableTiming);
        if (e == hipSuccess && i > 0) e = hipEventCreateWithFlags(&x->sc[i].end, hipEventDisableTiming);
    }
    if (e == hipSuccess) e = hipEventCreateWithFlags(&x->sc_static.end, hipEventDisableTiming);
    if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void**>(&x->h_counters), sizeof(unsigned long long) * kNumCounters);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&x->ev_search_end, hipEventDisableTiming);
    x->sc[0].end = x->ev_search_end;
    if (e == hipSuccess) e = hipEventCreateWithFlags(&x->ev_probes, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&x->ev_done, hipEventDisableTiming);
    for (int i = 0; e == hipSuccess && i < kMaxStage; ++i) {
        e = hipEventCreateWithFlags(&x->stage_free[i], hipEventDisableTiming);
        for (int sd = 0; e == hipSuccess && sd < kMaxSide; ++sd)
            e = hipEventCreateWithFlags(&x->stage_ready[i][sd], hipEventDisableTiming);
    }
    if (e != hipSuccess) {
        (void)hipGetLastError();
        int rc = fail(IVF_ERR_HIP, "index creation failed: %s", hipGetErrorString(e));
        ivf_index_destroy(x);
        return rc;
    }
    x->cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    // the static scratch array of ivf_search_noalloc: its address on this device, looked up once
    if (int rc = static_scratch_init(x->device)) {
        std::string msg = g_err;
        ivf_index_destroy(x);
        g_err = msg;
        return rc;
    }
    x->static_base = g_static[x->device].base;
    *out = x;
    return 0;
}

void ivf_index_destroy(ivf_index* x) {
    if (!x) return;
    (void)hipDeviceSynchronize();
    free_index_data(x);
    dfree(x->d_codebooks);
    for (int i = 0; i < kMaxSide; ++i)
        if (x->side[i]) (void)hipStreamDestroy(x->side[i]);
    if (x->move_stream) (void)hipStreamDestroy(x->move_stream);
    if (x->patch_stream) (void)hipStreamDestroy(x->patch_stream);
    if (x->pipe_scan) (void)hipStreamDestroy(x->pipe_scan);
    for (int i = 0; i < 2; ++i)
        if (x->ev_trial[i]) (void)hipEventDestroy(x->ev_trial[i]);
    for (int i = 0; i < 2; ++i)
        if (x->pipe_front[i]) (void)hipStreamDestroy(x->pipe_front[i]);
    for (int i = 0; i < kSets; ++i) {
        if (x->ev_front[i]) (void)hipEventDestroy(x->ev_front[i]);
        if (x->ev_scan[i]) (void)hipEventDestroy(x->ev_scan[i]);
        if (i > 0 && x->sc[i].end) (void)hipEventDestroy(x->sc[i].end);
    }
    if (x->sc_static.end) (void)hipEventDestroy(x->sc_static.end);
    if (x->h_counters) (void)hipHostFree(x->h_counters);
    if (x->ev_search_end) (void)hipEventDestroy(x->ev_search_end);
    for (hipEvent_t e : x->spare_events) (void)hipEventDestroy(e);
    if (x->ev_probes) (void)hipEventDestroy(x->ev_probes);
    if (x->ev_done) (void)hipEventDestroy(x->ev_done);
    for (int i = 0; i < kMaxStage; ++i) {
        for (int sd = 0; sd < kMaxSide; ++sd)
            if (x->stage_ready[i][sd]) (void)hipEventDestroy(x->stage_ready[i][sd]);
        if (x->stage_free[i]) (void)hipEventDestroy(x->stage_free[i]);
    }
    for (int sl = 0; sl < kTimingSlots; ++sl)
        for (int i = 0; i < kEvPerSearch; ++i)
            if (x->ev[sl][i]) (void)hipEventDestroy(x->ev[sl][i]);
    delete x;
}

int ivf_index_set_pq_codebooks(ivf_index* x, int d, int m, const float* codebooks) {
    if (!x || !codebooks) return fail(IVF_ERR_INVALID, "index or codebooks is NULL");
    if (x->uploading) return fail(IVF_ERR_INVALID, "codebooks cannot change during an upload");
    if (d <= 0 || m <= 0 || d % m != 0) return fail(IVF_ERR_INVALID, "d must be a positive multiple of m");
    if (m % 16 != 0 || m > kPqMaxM) return fail(IVF_ERR_LIMIT, "m must be a multiple of 16 and at most %d (got %d)", kPqMaxM, m);
    if (x->ready && x->dtype == IVF_PQ8) return fail(IVF_ERR_INVALID, "the index holds codes of the current codebooks: upload anew first");
    (void)hipDeviceSynchronize();
    dfree(x->d_codebooks);
    x->pq_m = x->pq_d = 0;
    size_t tot = 0;
    int rc;
    if ((rc = dalloc(x->d_codebooks, (size_t)256 * d, tot))) return rc;
    HIP_TRY(hipMemcpy(x->d_codebooks, codebooks, sizeof(float) * 256 * (size_t)d, hipMemcpyDefault));
    if (!x->pq_lds_set) {
        // a table of up to 128 KiB in LDS is beyond the default allowance of a workgroup
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(k_pq_scan), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    kPqMaxM * 1024));
        x->pq_lds_set = true;
    }
    x->pq_m = m;
    x->pq_d = d;
    return 0;
}

int ivf_index_upload_begin(ivf_index* x, int d, int64_t nlist, int64_t n, const float* centroids,
                           int dtype, const int64_t* list_offsets) {
    if (!x) return fail(IVF_ERR_INVALID, "index is NULL");
    if (!centroids || !list_offsets) return fail(IVF_ERR_INVALID, "centroids or list_offsets is NULL");
    if (dtype != IVF_FP32 && dtype != IVF_FP16 && dtype != IVF_INT8 && dtype != IVF_PQ8)
        return fail(IVF_ERR_INVALID, "dtype must be IVF_FP32, IVF_FP16, IVF_INT8 or IVF_PQ8");
    if (dtype == IVF_PQ8 && (!x->d_codebooks || x->pq_d != d))
        return fail(IVF_ERR_INVALID, "IVF_PQ8 needs codebooks for this dimension first (ivf_index_set_pq_codebooks)");
    if (d <= 0 || nlist <= 0 || n < 0) return fail(IVF_ERR_INVALID, "d, nlist must be positive and n non-negative");
    if (d % 8 != 0 || d > 4096) return fail(IVF_ERR_LIMIT, "d must be a multiple of 8 and at most 4096 (got %d)", d);
    if (dtype == IVF_INT8 && d % 16 != 0) return fail(IVF_ERR_LIMIT, "d must be a multiple of 16 for int8 storage (got %d)", d);
    if (n >= (int64_t)1 << 32 || nlist >= (int64_t)1 << 28)
        return fail(IVF_ERR_LIMIT, "n must be below 2^32 and nlist below 2^28");
    (void)hipDeviceSynchronize();
    free_index_data(x);
    x->d = d; x->dtype = dtype; x->es = dtype == IVF_FP16 ? 2 : (dtype == IVF_INT8 || dtype == IVF_PQ8) ? 1 : 4;
    x->nlist = nlist; x->n = n;
    x->tail_bytes = dtype == IVF_INT8 ? 4 : 0;       // int8 records end with their fp32 scale
    x->row_bytes = dtype == IVF_PQ8 ? (size_t)x->pq_m : (size_t)d * x->es + x->tail_bytes;
    x->block_bytes = x->row_bytes * kLanes;
    try {
        x->offsets.assign((size_t)nlist + 1, 0);
        x->blk_off.assign((size_t)nlist + 1, 0);
        x->len.assign((size_t)nlist, 0);
        x->nblk.assign((size_t)nlist, 0);
        x->dev_ptr.assign((size_t)nlist, nullptr);
        x->host_ptr.assign((size_t)nlist, nullptr);
        x->loc.assign((size_t)nlist, Loc());
    } catch (const std::bad_alloc&) {
        return fail(IVF_ERR_OOM_HOST, "out of host memory for the list tables");
    }
    HIP_TRY(hipMemcpy(x->offsets.data(), list_offsets, sizeof(int64_t) * ((size_t)nlist + 1), hipMemcpyDefault));
    if (x->offsets[0] != 0 || x->offsets[(size_t)nlist] != n)
        return fail(IVF_ERR_INVALID, "list_offsets must start at 0 and end at n");
    x->max_len = 0;
    for (int64_t l = 0; l < nlist; ++l) {
        int64_t ln = x->offsets[l + 1] - x->offsets[l];
        if (ln < 0) return fail(IVF_ERR_INVALID, "list_offsets must be non-decreasing (list %lld)", (long long)l);
        if (ln > (int64_t)65535 * kLanes) return fail(IVF_ERR_LIMIT, "list %lld longer than %d vectors", (long long)l, 65535 * kLanes);
        x->len[l] = (int32_t)ln;
        x->nblk[l] = (int32_t)((ln + kLanes - 1) / kLanes);
        x->blk_off[l + 1] = x->blk_off[l] + x->nblk[l];
        x->max_len = std::max(x->max_len, ln);
    }
    x->total_blocks = x->blk_off[(size_t)nlist];
    {
        std::vector<int32_t> srt(x->nblk);
        std::sort(srt.begin(), srt.end(), std::greater<int32_t>());
        size_t m = std::min<size_t>(srt.size(), kMaxK);
        x->top_nblk_prefix.assign(m + 1, 0);
        for (size_t i = 0; i < m; ++i) x->top_nblk_prefix[i + 1] = x->top_nblk_prefix[i] + srt[i];
    }
    size_t tot = 0;
    int rc;
    const int cstep = (d + kCoarseKT - 1) / kCoarseKT;
    const size_t ctiles = ((size_t)nlist + 31) / 32;
    if ((rc = dalloc(x->d_centroids, ctiles * cstep * 1024, tot))) return rc;    // tiled for k_coarse
    if ((rc = dalloc(x->d_offsets, (size_t)nlist + 1, tot))) return rc;
    if ((rc = dalloc(x->d_len, (size_t)nlist, tot))) return rc;
    if ((rc = dalloc(x->d_nblk, (size_t)nlist, tot))) return rc;
    if ((rc = dalloc(x->d_list_ptr, (size_t)nlist, tot))) return rc;
    if ((rc = dalloc(x->d_ids_pos, (size_t)n, tot))) return rc;
    if ((rc = dalloc(x->d_hits, (size_t)nlist, tot))) return rc;
    HIP_TRY(hipMemset(x->d_hits, 0, sizeof(uint32_t) * (size_t)nlist));
    {
        hipError_t e = hipHostMalloc(reinterpret_cast<void**>(&x->h_list_ptr), sizeof(void*) * (size_t)nlist);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            x->h_list_ptr = nullptr;
            return fail(IVF_ERR_OOM_HOST, "pinned mirror of the list table: %s", hipGetErrorString(e));
        }
    }
    {
        // segment size: a sixteenth of the index, between 64 MiB and the "segment_mb" option
        size_t total_bytes = (size_t)x->total_blocks * x->block_bytes;
        size_t seg_bytes = std::min<size_t>((size_t)x->opt_segment_mb << 20, std::max<size_t>((size_t)64 << 20, total_bytes / 16));
        size_t max_nb = 1;
        for (int64_t l = 0; l < nlist; ++l) max_nb = std::max<size_t>(max_nb, (size_t)x->nblk[l]);
        x->dpool = Pool(); x->hpool = Pool();
        x->dpool.alloc = hbm_alloc; x->dpool.dealloc = hbm_free;
        x->hpool.alloc = pinned_alloc; x->hpool.dealloc = pinned_free;
        x->dpool.block_bytes = x->hpool.block_bytes = x->block_bytes;
        x->dpool.seg_blocks = x->hpool.seg_blocks = std::max<size_t>(max_nb, seg_bytes / x->block_bytes);
        size_t left = (size_t)x->total_blocks;
        for (int64_t l = 0; l < nlist; ++l) {
            const size_t nb = (size_t)x->nblk[l];
            Loc& c = x->loc[l];
            c.tier = 0;
            if (!nb) continue;
            // the last segment is no larger than what is still to be placed
            x->dpool.seg_blocks = std::max<size_t>(max_nb, std::min(x->dpool.seg_blocks, left));
            if (!pool_alloc(x->dpool, nb, c.seg, c.off, true)) {
                pool_free_all(x->dpool);
                return fail(IVF_ERR_OOM_DEVICE, "out of device memory for the list data (%zu bytes in all)", total_bytes);
            }
            left -= nb;
        }
        x->dpool.seg_blocks = x->hpool.seg_blocks;
    }
    {
        float* raw = nullptr;
        size_t unused = 0;
        if ((rc = dalloc(raw, (size_t)nlist * d, unused))) return rc;
        hipError_t e = hipMemcpy(raw, centroids, sizeof(float) * (size_t)nlist * d, hipMemcpyDefault);
        if (e == hipSuccess) {
            const size_t nv = ctiles * cstep * 256;
            hipLaunchKernelGGL(k_tile_centroids, dim3((unsigned)((nv + 255) / 256)), dim3(256), 0, 0, raw, x->d_centroids,
                               (int)nlist, d, cstep, nv);
            e = hipGetLastError();
            if (e == hipSuccess) e = hipDeviceSynchronize();
        }
        dfree(raw);
        HIP_TRY(e);
    }
    HIP_TRY(hipMemcpy(x->d_offsets, x->offsets.data(), sizeof(int64_t) * ((size_t)nlist + 1), hipMemcpyHostToDevice));
    HIP_TRY(hipMemcpy(x->d_len, x->len.data(), sizeof(int32_t) * (size_t)nlist, hipMemcpyHostToDevice));
    HIP_TRY(hipMemcpy(x->d_nblk, x->nblk.data(), sizeof(int32_t) * (size_t)nlist, hipMemcpyHostToDevice));
    if ((rc = upload_list_ptr_table(x))) return rc;
    x->resident_lists = nlist;
    x->next_list = 0;
    x->uploading = true;
    return 0;
}

int ivf_index_upload_lists(ivf_index* x, int64_t list_begin, int64_t list_end, const void* vectors,
                           const int64_t* ids) {
    if (!x || !x->uploading) return fail(IVF_ERR_INVALID, "upload_lists without upload_begin");
    if (list_begin != x->next_list || list_end < list_begin || list_end > x->nlist)
        return fail(IVF_ERR_INVALID, "pieces must cover the lists in ascending order without gaps (expected list %lld)",
                    (long long)x->next_list);
    const int64_t r0 = x->offsets[list_begin], r1 = x->offsets[list_end];
    const int64_t rows = r1 - r0;
    if (rows > 0 && (!vectors || !ids)) return fail(IVF_ERR_INVALID, "vectors or ids is NULL");
    if (rows > 0) {
        HIP_TRY(hipMemcpy(x->d_ids_pos + r0, ids, sizeof(int64_t) * (size_t)rows, hipMemcpyDefault));
        const bool on_dev = is_device_ptr(vectors);
        char* tmp = nullptr;
        size_t tmp_bytes = 0;
        if (!on_dev) {
            tmp_bytes = std::max<size_t>((size_t)256 << 20, (size_t)x->max_len * x->row_bytes);
            tmp_bytes = std::min(tmp_bytes, (size_t)rows * x->row_bytes);
            hipError_t e = hipMalloc(reinterpret_cast<void**>(&tmp), tmp_bytes);
            if (e != hipSuccess) {
                (void)hipGetLastError();
                return fail(IVF_ERR_OOM_DEVICE, "upload staging of %zu bytes: %s", tmp_bytes, hipGetErrorString(e));
            }
        }
        int64_t lb = list_begin;
        int rc = 0;
        while (lb < list_end && rc == 0) {
            int64_t le = lb;
            if (on_dev) {
                le = list_end;
            } else {
                while (le < list_end && (size_t)(x->offsets[le + 1] - x->offsets[lb]) * x->row_bytes <= tmp_bytes) ++le;
            }
            const int64_t pr = x->offsets[le] - x->offsets[lb];
            int32_t maxnb = 0;
            for (int64_t l = lb; l < le; ++l) maxnb = std::max(maxnb, x->nblk[l]);
            if (pr > 0) {
                const char* src = static_cast<const char*>(vectors) + (size_t)(x->offsets[lb] - r0) * x->row_bytes;
                hipError_t e = hipSuccess;
                if (!on_dev) {
                    e = hipMemcpy(tmp, src, (size_t)pr * x->row_bytes, hipMemcpyHostToDevice);
                    src = tmp;
                }
                if (e == hipSuccess) {
                    dim3 grid((unsigned)(le - lb), (unsigned)maxnb);
                    hipLaunchKernelGGL(k_relayout, grid, dim3(256), 0, 0, src, x->d_offsets, x->d_list_ptr, lb,
                                       (int)x->row_bytes, x->tail_bytes);
                    e = hipGetLastError();
                    if (e == hipSuccess) e = hipDeviceSynchronize();
                }
                if (e != hipSuccess) {
                    (void)hipGetLastError();
                    rc = fail(IVF_ERR_HIP, "re-layout of lists [%lld,%lld) failed: %s", (long long)lb, (long long)le,
                              hipGetErrorString(e));
                }
            }
            lb = le;
        }
        if (tmp) (void)hipFree(tmp);
        if (rc) return rc;
    }
    x->next_list = list_end;
    return 0;
}

int ivf_index_upload_end(ivf_index* x) {
    if (!x || !x->uploading) return fail(IVF_ERR_INVALID, "upload_end without upload_begin");
    if (x->next_list != x->nlist)
        return fail(IVF_ERR_INVALID, "only %lld of %lld lists were uploaded", (long long)x->next_list, (long long)x->nlist);
    size_t tot = 0;
    int rc;
    const size_t n = (size_t)x->n;
    uint32_t* pos_in = nullptr;
    uint32_t* pos_sorted = nullptr;
    if ((rc = dalloc(x->d_id_sorted, n, tot))) return rc;
    if ((rc = dalloc(x->d_rank_of_pos, n, tot))) return rc;
    if ((rc = dalloc(pos_in, n, tot))) return rc;
    if ((rc = dalloc(pos_sorted, n, tot))) { dfree(pos_in); return rc; }
    if (n > 0) {
        const unsigned g = (unsigned)((n + 255) / 256);
        hipLaunchKernelGGL(k_iota_u32, dim3(g), dim3(256), 0, 0, pos_in, n);
        int e = ivf_internal_sort_pairs(x->d_ids_pos, x->d_id_sorted, pos_in, pos_sorted, n, 0);
        if (e == 0) {
            hipLaunchKernelGGL(k_scatter_rank, dim3(g), dim3(256), 0, 0, pos_sorted, x->d_rank_of_pos, n);
            e = (int)hipDeviceSynchronize();
        }
        if (e != 0) {
            (void)hipGetLastError();
            dfree(pos_in); dfree(pos_sorted);
            return fail(e == (int)hipErrorOutOfMemory ? IVF_ERR_OOM_DEVICE : IVF_ERR_HIP, "id ranking failed: %s",
                        hipGetErrorString((hipError_t)e));
        }
    }
    dfree(pos_in);
    dfree(pos_sorted);
    dfree(x->d_ids_pos);
    if ((rc = upload_list_ptr_table(x))) return rc;
    x->uploading = false;
    x->ready = true;
    return 0;
}

int ivf_index_upload(ivf_index* x, int d, int64_t nlist, int64_t n, const float* centroids,
                     const void* vectors, int dtype, const int64_t* ids, const int64_t* list_offsets) {
    int rc = ivf_index_upload_begin(x, d, nlist, n, centroids, dtype, list_offsets);
    if (rc) return rc;
    if ((rc = ivf_index_upload_lists(x, 0, nlist, vectors, ids))) return rc;
    return ivf_index_upload_end(x);
}

int ivf_set_device_budget(ivf_index* x, int64_t bytes) {
    int rc = check_ready(x);
    if (rc) return rc;
    if (bytes < 0) return fail(IVF_ERR_INVALID, "budget must be non-negative");
    if ((rc = moves_drain(x, true))) return rc;       // an earlier asynchronous change ends where it is
    HIP_TRY(hipDeviceSynchronize());
    if ((rc = budget_plan(x, bytes))) return rc;
    if ((rc = moves_drain(x, false))) return rc;
    if (x->move_rc) return fail(x->move_rc, "%s", x->move_msg.c_str());
    if (x->resident_lists < x->nlist) {
        if (!x->opt_host_direct && (rc = ensure_staging(x))) return rc;
    } else {
        HIP_TRY(hipDeviceSynchronize());
        free_staging(x);
    }
    return 0;
}

int ivf_set_device_budget_async(ivf_index* x, int64_t bytes) {
    int rc = check_ready(x);
    if (rc) return rc;
    if (bytes < 0) return fail(IVF_ERR_INVALID, "budget must be non-negative");
    if ((rc = moves_drain(x, true))) return rc;       // copies of an earlier change that are under way finish first
    HIP_TRY(hipDeviceSynchronize());                  // searches issued so far are not tracked: let them end
    if ((rc = budget_plan(x, bytes))) return rc;
    if ((rc = moves_advance(x))) return rc;
    if (x->move_rc) return fail(x->move_rc, "%s", x->move_msg.c_str());
    return 0;
}

int ivf_budget_progress(ivf_index* x, int64_t* pending_lists, int64_t* pending_bytes, int* busy) {
    int rc = check_ready(x);
    if (rc) return rc;
    if (moves_active(x) && (rc = moves_advance(x))) return rc;
    int64_t pl = 0, pb = 0;
    count_pending(x, pl, pb);
    if (pending_lists) *pending_lists = pl;
    if (pending_bytes) *pending_bytes = pb;
    if (busy) *busy = moves_active(x) ? 1 : 0;
    if (x->move_rc) return fail(x->move_rc, "%s", x->move_msg.c_str());
    return 0;
}

int ivf_budget_wait(ivf_index* x) {
    int rc = check_ready(x);
    if (rc) return rc;
    if ((rc = moves_drain(x, false))) return rc;
    if (x->move_rc) return fail(x->move_rc, "%s", x->move_msg.c_str());
    return 0;
}

int ivf_search(ivf_index* x, const float* queries, int64_t nq, int nprobe, int k, int64_t* out_ids,
               float* out_scores, void* stream) {
    SearchCtx c;
    int rc = search_args(x, queries, nq, nprobe, k, out_ids, out_scores, c);
    if (rc) return rc < 0 ? rc : 0;          // 1: nothing to do
    hipStream_t st = static_cast<hipStream_t>(stream);
    Scratch& s = x->sc[0];
    if ((rc = order_after_last_use(s, st, st))) return rc;
    if ((rc = search_prologue(x, st, c))) return rc;
    if ((rc = ensure_scratch(x, s, c.nq, c.nprobe, c.offload, c.q_host))) {
        // a failed growth leaves some buffers freed: drop all of them so that the sizes on
        // record match what exists (the next search allocates afresh); the error message stays
        std::string msg = g_err;
        (void)hipDeviceSynchronize();
        free_scratch(s);
        g_err = msg;
        return rc;
    }
    return search_serial(x, s, c, st);
}

// A single wavefront that runs for about `ticks` periods of the 100 MHz wall clock and then
// ends; the iteration cap ends it whatever the clock does.
__global__ void k_spin(long long ticks, unsigned* __restrict__ sink) {
    const long long t0 = wall_clock64();
    unsigned n = 0;
    while (wall_clock64() - t0 < ticks && n < (1u << 24)) ++n;
    if (n == 0xffffffffu) sink[0] = n;       // never true: keeps the loop
}

__global__ void k_nothing() {}

// Does a kernel on `b` run while one on `a` is still running?  (Both streams idle.)  A
// kernel of about 60 us goes to `a`, an empty one to `b`; the streams share a hardware
// queue if the empty one ends after the long one.
int streams_run_side_by_side(ivf_index* x, hipStream_t a, hipStream_t b, bool& yes) {
    hipLaunchKernelGGL(k_spin, dim3(1), dim3(64), 0, a, (long long)6000, (unsigned*)x->h_counters);
    HIP_TRY(hipEventRecord(x->ev_trial[0], a));
    hipLaunchKernelGGL(k_nothing, dim3(1), dim3(64), 0, b);
    HIP_TRY(hipEventRecord(x->ev_trial[1], b));
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipEventSynchronize(x->ev_trial[0]));
    HIP_TRY(hipEventSynchronize(x->ev_trial[1]));
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, x->ev_trial[1], x->ev_trial[0]));   // > 0: b's ended first
    yes = ms > 0.02f;
    return 0;
}

// Picks the library's three streams for queued searches (two for front stages, one for the
// scans) so that they and the caller's stream `st` run side by side, i.e. sit on different
// hardware queues: new streams are made one by one and tried against the caller's stream
// and those picked so far; those that share a queue with one of them are destroyed again
// at the end.  Done once per index, at the first queued search that finds `st` idle (work
// already on it would make every trial look like a shared queue) or, failing that, at the
// eighth, which waits for the device; a later call on another stream keeps the choice.
// When a dozen streams do not yield three, the rest are taken as they come: the searches
// are then correct and slower.
int pick_pipe_streams(ivf_index* x, hipStream_t st) {
    if (x->pipe_picked) return 0;
    int rc;
    const bool idle = hipStreamQuery(st) == hipSuccess;
    (void)hipGetLastError();
    if (!idle && ++x->pipe_pick_tries < 8) {
        // not now: make do with streams as they come, and try again at the next search
        for (hipStream_t* s : {&x->pipe_front[0], &x->pipe_front[1], &x->pipe_scan})
            if ((rc = need_stream(*s))) return rc;
        return 0;
    }
    for (int i = 0; i < 2; ++i)
        if (!x->ev_trial[i]) HIP_TRY(hipEventCreate(&x->ev_trial[i]));
    // earlier searches may still run on streams made before: trials need them idle
    HIP_TRY(hipDeviceSynchronize());
    std::vector<hipStream_t> picked, spare, tried;
    for (hipStream_t s : {x->pipe_front[0], x->pipe_front[1], x->pipe_scan})
        if (s) spare.push_back(s);               // made by a call that could not run the trials
    x->pipe_front[0] = x->pipe_front[1] = x->pipe_scan = nullptr;
    int rc_trials = 0;
    for (int n = 0; n < 12 && picked.size() < 3 && !rc_trials; ++n) {
        hipStream_t c = nullptr;
        if (!spare.empty()) { c = spare.back(); spare.pop_back(); }
        else if ((rc_trials = need_stream(c))) break;
        bool ok = true;
        rc_trials = streams_run_side_by_side(x, st, c, ok);
        for (size_t i = 0; !rc_trials && ok && i < picked.size(); ++i)
            rc_trials = streams_run_side_by_side(x, picked[i], c, ok);
        (ok && !rc_trials ? picked : tried).push_back(c);
    }
    // whatever happened, the index ends up owning three streams (or as many as could be
    // made) and nothing else
    for (hipStream_t s : spare) tried.push_back(s);
    while (picked.size() < 3 && !tried.empty()) { picked.push_back(tried.back()); tried.pop_back(); }
    for (hipStream_t s : tried) (void)hipStreamDestroy(s);
    hipStream_t* slots[3] = {&x->pipe_scan, &x->pipe_front[0], &x->pipe_front[1]};
    for (size_t i = 0; i < picked.size(); ++i) *slots[i] = picked[i];
    if (rc_trials) return rc_trials;
    for (hipStream_t* s : slots)
        if ((rc = need_stream(*s))) return rc;
    x->pipe_picked = true;
    x->pipe_caller = st;
    return 0;
}

int ivf_search_queued(ivf_index* x, const float* queries, int64_t nq, int nprobe, int k, int64_t* out_ids,
                      float* out_scores, void* stream, void* queries_ready) {
    SearchCtx c;
    int rc = search_args(x, queries, nq, nprobe, k, out_ids, out_scores, c);
    if (rc) return rc < 0 ? rc : 0;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipEvent_t ready = static_cast<hipEvent_t>(queries_ready);
    // Budget changes under way, the staged host-list mode and per-stage timing keep a search
    // on one stream; it then starts behind the queries like any other work of that stream.
    // So does a search whose scan is bounded by a few tens of microseconds: the overlap
    // cannot repay the dozen extra stream and event calls it takes.
    const uint64_t bound_bytes = (uint64_t)block_bound(x, c.nq, c.nprobe) * x->block_bytes;
    const bool tiny = bound_bytes < ((uint64_t)x->opt_queue_min_mb << 20);
    // And so does any search over an index with host-resident lists: its scan is bound by
    // PCIe, there is nothing to gain, and under a scan whose wavefronts sit on PCIe reads
    // for milliseconds the final selection of the search before would wait that long for
    // room on a compute unit (8 ms at C4), i.e. its results would be late.
    const bool serial = tiny || stream_is_capturing(st) || moves_active(x) || x->resident_lists < x->nlist || x->timing == 1;
    const int p = serial ? 0 : x->next_set;
    // Under a scan the front kernels (chains of dependent loads) run several times slower
    // than alone.  Behind a short scan (a few hundred microseconds) one search's worth of
    // them no longer fits, and the searches' front stages alternate between two streams;
    // behind a long scan a second stream only takes more from the scan.
    const int fronts = x->opt_queue_fronts ? (int)x->opt_queue_fronts : bound_bytes < ((uint64_t)4 << 30) ? 2 : 1;
    if (!serial && (rc = pick_pipe_streams(x, st))) return rc;
    hipStream_t own_front = x->pipe_front[x->queued_count % (uint64_t)fronts];
    hipStream_t first = serial ? st : own_front;
    Scratch& s = x->sc[p];
    if ((rc = order_after_last_use(s, st, first))) return rc;
    if (serial) {
        if (ready) HIP_TRY(hipStreamWaitEvent(st, ready, 0));
        if ((rc = search_prologue(x, st, c))) return rc;
    }
    if ((rc = ensure_scratch(x, s, c.nq, c.nprobe, c.offload, c.q_host))) {
        std::string msg = g_err;
        (void)hipDeviceSynchronize();
        free_scratch(s);
        g_err = msg;
        return rc;
    }
    if (serial) return search_serial(x, s, c, st);

    // By stage: the front stages of consecutive searches alternate between two streams of
    // the library, every scan runs on a third behind the scan of the search before, and the
    // final selection runs on the caller's stream, where the results are wanted (four
    // streams in all: a process has four hardware queues, and streams that share one run
    // one after the other).  Events carry a search from stage to stage and hand its scratch
    // set (one of kSets, taken in turn) to the search that uses it next.
    hipStream_t front = first, scan = x->pipe_scan;
    x->queued_count += 1;
    const int tm = x->timing;                  // 0 or 2 here
    hipEvent_t* evs = x->ev[x->timed_searches % kTimingSlots];
    search_set_pruning(x, c);
    if (ready) HIP_TRY(hipStreamWaitEvent(front, ready, 0));
    if ((rc = stage_queries(x, s, c, front))) return rc;
    enqueue_coarse(x, s, c, front);
    enqueue_probe_select(x, s, c, front, true);
    enqueue_regroup(x, s, c, front, true);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipEventRecord(x->ev_front[p], front));
    HIP_TRY(hipStreamWaitEvent(scan, x->ev_front[p], 0));
    // with timing on, the event behind the scan also tells the final selection to start:
    // every record on the scan's stream is a gap between two scans
    hipEvent_t scan_done = tm ? evs[4] : x->ev_scan[p];
    c.scan_start = tm ? evs[3] : nullptr;
    c.scan_stop = scan_done;
    enqueue_scan(x, s, c, scan);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamWaitEvent(st, scan_done, 0));
    enqueue_final_select(x, s, c, st, true);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipEventRecord(s.end, st));
    s.end_recorded = true;
    x->next_set = (p + 1) % kSets;
    search_epilogue(x, s, c, st, true);
    if (tm) {
        x->ev_queued[x->timed_searches % kTimingSlots] = true;
        x->timed_searches += 1;
    }
    return 0;
}

int ivf_search_noalloc(ivf_index* x, const float* queries, int64_t nq, int nprobe, int k, int64_t* out_ids,
                       float* out_scores, void* stream) {
    SearchCtx c;
    int rc = search_args(x, queries, nq, nprobe, k, out_ids, out_scores, c);
    if (rc) return rc < 0 ? rc : 0;
    if (moves_active(x))
        return fail(IVF_ERR_INVALID, "ivf_search_noalloc: a budget change is under way (it allocates and frees pool segments)");
    if (c.offload)
        return fail(IVF_ERR_INVALID, "ivf_search_noalloc: the staged host-list mode needs staging buffers; use host_direct = 1");
    if (!x->static_base) return fail(IVF_ERR_HIP, "ivf_search_noalloc: the static scratch array has no address on this device");
    Scratch& s = x->sc_static;
    const size_t need = carve_scratch(x, c.nq, c.nprobe, c.q_host, x->static_base, kStaticScratchBytes, s);
    if (need > kStaticScratchBytes)
        return fail(IVF_ERR_LIMIT, "ivf_search_noalloc: this search needs %zu bytes of scratch, the static array holds %zu "
                    "(nq*nlist coarse scores plus 292 bytes per 64-vector block of nq times the nprobe longest lists)",
                    need, (size_t)kStaticScratchBytes);
    hipStream_t st = static_cast<hipStream_t>(stream);
    // every index on this GPU shares the array: this search starts behind the last one that used it
    StaticScratchDevice& dv = g_static[x->device];
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (dv.used) HIP_TRY(hipStreamWaitEvent(st, dv.last_use, 0));
    rc = search_serial(x, s, c, st);
    if (hipEventRecord(dv.last_use, st) == hipSuccess) dv.used = true;
    else { (void)hipGetLastError(); (void)hipStreamSynchronize(st); }
    return rc;
}

int ivf_get_info(ivf_index* x, ivf_info* out) {
    int rc = check_ready(x);
    if (rc) return rc;
    if (!out) return fail(IVF_ERR_INVALID, "out is NULL");
    out->d = x->d; out->dtype = x->dtype; out->nlist = x->nlist; out->n = x->n;
    out->max_list_len = x->max_len;
    out->index_bytes = (int64_t)((size_t)x->total_blocks * x->block_bytes);
    int64_t dev = 0;
    for (int64_t l = 0; l < x->nlist; ++l)
        if (x->dev_ptr[l]) dev += (int64_t)x->nblk[l] * (int64_t)x->block_bytes;
    out->device_list_bytes = dev;
    out->host_list_bytes = out->index_bytes - dev;
    out->resident_lists = x->resident_lists;
    out->scratch_bytes = 0;
    for (int p = 0; p < kSets; ++p) out->scratch_bytes += (int64_t)x->sc[p].bytes;
    out->device_pool_bytes = (int64_t)(x->dpool.allocated_blocks() * x->block_bytes);
    out->host_pool_bytes = (int64_t)(x->hpool.allocated_blocks() * x->block_bytes);
    out->moved_h2d_bytes = x->moved_h2d;
    out->moved_d2h_bytes = x->moved_d2h;
    out->moved_d2d_bytes = x->moved_d2d;
    return 0;
}

int ivf_debug_last_probes(ivf_index* x, int32_t* out_lists, void* stream) {
    int rc = check_ready(x);
    if (rc) return rc;
    if (!out_lists || x->last_nq == 0 || !x->last_sc) return fail(IVF_ERR_INVALID, "no search yet or out_lists is NULL");
    HIP_TRY(hipMemcpyAsync(out_lists, x->last_sc->probes, sizeof(int32_t) * (size_t)x->last_nq * x->last_nprobe,
                           hipMemcpyDeviceToDevice, static_cast<hipStream_t>(stream)));
    return 0;
}

int ivf_debug_last_coarse(ivf_index* x, float* out_scores, void* stream) {
    int rc = check_ready(x);
    if (rc) return rc;
    if (!out_scores || x->last_nq == 0 || !x->last_sc) return fail(IVF_ERR_INVALID, "no search yet or out_scores is NULL");
    HIP_TRY(hipMemcpyAsync(out_scores, x->last_sc->S, sizeof(float) * (size_t)x->last_nq * (size_t)x->nlist,
                           hipMemcpyDeviceToDevice, static_cast<hipStream_t>(stream)));
    return 0;
}

int ivf_debug_read_list(ivf_index* x, int64_t list, void* out_vectors, int64_t* out_ids, int64_t* len) {
    int rc = check_ready(x);
    if (rc) return rc;
    if (list < 0 || list >= x->nlist) return fail(IVF_ERR_INVALID, "list out of range");
    HIP_TRY(hipDeviceSynchronize());
    const int64_t ln = x->len[list];
    if (len) *len = ln;
    if (ln == 0) return 0;
    const size_t bytes = (size_t)x->nblk[list] * x->block_bytes;
    if (out_vectors) {
        char* blk = nullptr;
        char* rows = nullptr;
        const char* src = x->dev_ptr[list];
        hipError_t e = hipMalloc(reinterpret_cast<void**>(&rows), (size_t)ln * x->row_bytes);
        if (e == hipSuccess && !src) {
            e = hipMalloc(reinterpret_cast<void**>(&blk), bytes);
            if (e == hipSuccess) e = hipMemcpy(blk, x->host_ptr[list], bytes, hipMemcpyHostToDevice);
            src = blk;
        }
        if (e == hipSuccess) {
            hipLaunchKernelGGL(k_unlayout, dim3((unsigned)x->nblk[list]), dim3(256), 0, 0, src, ln, (int)x->row_bytes,
                               x->tail_bytes, rows);
            e = hipGetLastError();
        }
        if (e == hipSuccess) e = hipMemcpy(out_vectors, rows, (size_t)ln * x->row_bytes, hipMemcpyDeviceToHost);
        if (rows) (void)hipFree(rows);
        if (blk) (void)hipFree(blk);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            return fail(IVF_ERR_HIP, "read-back failed: %s", hipGetErrorString(e));
        }
    }
    if (out_ids) {
        int64_t* tmp = nullptr;
        hipError_t e = hipMalloc(reinterpret_cast<void**>(&tmp), sizeof(int64_t) * (size_t)ln);
        if (e == hipSuccess) {
            hipLaunchKernelGGL(k_gather_ids, dim3((unsigned)((ln + 255) / 256)), dim3(256), 0, 0, x->d_id_sorted,
                               x->d_rank_of_pos, x->offsets[list], ln, tmp);
            e = hipMemcpy(out_ids, tmp, sizeof(int64_t) * (size_t)ln, hipMemcpyDeviceToHost);
        }
        if (tmp) (void)hipFree(tmp);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            return fail(IVF_ERR_HIP, "id read-back failed: %s", hipGetErrorString(e));
        }
    }
    return 0;
}

int ivf_last_search_stats(ivf_index* x, ivf_search_stats* out) {
    int rc = check_ready(x);
    if (rc) return rc;
    if (!out || x->last_nq == 0 || !x->last_sc) return fail(IVF_ERR_INVALID, "no search yet or out is NULL");
    if (x->last_sc->end_recorded) HIP_TRY(hipEventSynchronize(x->last_sc->end));
    else HIP_TRY(hipDeviceSynchronize());           // the search was captured into a graph: no event of its own
    if (!x->last_offload) {
        const unsigned long long* hc = x->h_counters;
        HIP_TRY(hipMemcpy(x->h_counters, x->last_sc->counters, sizeof(unsigned long long) * kNumCounters, hipMemcpyDeviceToHost));
        ivf_search_stats t = {};
        t.pairs = (int64_t)hc[kCntPairs];
        t.unique_lists = (int64_t)hc[kCntUnique];
        t.scanned_vectors = (int64_t)hc[kCntVectors];
        t.scan_bytes = t.scanned_vectors * (int64_t)x->row_bytes;
        t.scan_bytes_resident = (int64_t)hc[kCntVectorsResident] * (int64_t)x->row_bytes;
        t.scan_bytes_streamed = t.scan_bytes - t.scan_bytes_resident;
        t.scan_items = (int64_t)hc[kCntItems];
        x->last_stats = t;
    }
    *out = x->last_stats;
    return 0;
}

int ivf_set_timing(ivf_index* x, int enable) {
    if (!x) return fail(IVF_ERR_INVALID, "index is NULL");
    if (enable && !x->ev_created) {
        for (int sl = 0; sl < kTimingSlots; ++sl)
            for (int i = 0; i < kEvPerSearch; ++i) HIP_TRY(hipEventCreate(&x->ev[sl][i]));
        x->ev_created = true;
    }
    if (enable < 0 || enable > 2) return fail(IVF_ERR_INVALID, "timing level must be 0, 1 or 2");
    x->timing = enable;
    x->timed_searches = 0;
    return 0;
}

int ivf_get_stage_ms(ivf_index* x, int back, float* ms) {
    int rc = check_ready(x);
    if (rc) return rc;
    if (!ms) return fail(IVF_ERR_INVALID, "ms is NULL");
    if (back < 0 || back >= kTimingSlots || back >= x->timed_searches)
        return fail(IVF_ERR_INVALID, "no timed search %d calls back (kept: %d)", back, kTimingSlots);
    const int slot = (int)((x->timed_searches - 1 - back) % kTimingSlots);
    hipEvent_t* evs = x->ev[slot];
    for (int i = 0; i < IVF_NUM_STAGES; ++i) ms[i] = 0.f;
    if (x->ev_queued[slot]) {                // a queued search: events around its scan only
        HIP_TRY(hipEventSynchronize(evs[4]));
        HIP_TRY(hipEventElapsedTime(&ms[IVF_STAGE_SCAN], evs[3], evs[4]));
        ms[IVF_STAGE_TOTAL] = ms[IVF_STAGE_SCAN];
        return 0;
    }
    if (x->timing == 2) {                    // only the scan and streaming stages were recorded
        HIP_TRY(hipEventSynchronize(evs[5]));
        HIP_TRY(hipEventElapsedTime(&ms[IVF_STAGE_SCAN], evs[3], evs[4]));
        HIP_TRY(hipEventElapsedTime(&ms[IVF_STAGE_STREAM], evs[4], evs[5]));
        HIP_TRY(hipEventElapsedTime(&ms[IVF_STAGE_TOTAL], evs[3], evs[5]));
        return 0;
    }
    HIP_TRY(hipEventSynchronize(evs[6]));
    for (int i = 0; i < 6; ++i) HIP_TRY(hipEventElapsedTime(&ms[i], evs[i], evs[i + 1]));
    HIP_TRY(hipEventElapsedTime(&ms[IVF_STAGE_TOTAL], evs[0], evs[6]));
    return 0;
}

int ivf_debug_copy(void* dst, const void* src, int64_t bytes, void* stream) {
    if (!dst || !src || bytes < 0 || bytes % 16 != 0) return fail(IVF_ERR_INVALID, "dst/src NULL or bytes not a multiple of 16");
    if (bytes == 0) return 0;
    const size_t n = (size_t)bytes / 16;
    const unsigned grid = (unsigned)std::min<size_t>((n + 255) / 256, 256 * 32);
    hipLaunchKernelGGL(k_copy_u4, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<u4*>(dst), static_cast<const u4*>(src), n);
    HIP_TRY(hipGetLastError());
    return 0;
}

int ivf_debug_read(const void* src, int64_t bytes, void* sink, void* stream) {
    if (!src || !sink || bytes < 0 || bytes % 98304 != 0)
        return fail(IVF_ERR_INVALID, "src/sink NULL or bytes not a multiple of 98304");
    if (bytes == 0) return 0;
    const size_t ntiles = (size_t)bytes / 98304;
    hipLaunchKernelGGL(k_read_tiles, dim3((unsigned)((ntiles + 3) / 4)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u4*>(src), ntiles, static_cast<unsigned*>(sink));
    HIP_TRY(hipGetLastError());
    return 0;
}

int ivf_set_option(ivf_index* x, const char* name, int64_t value) {
    if (!x || !name) return fail(IVF_ERR_INVALID, "index or name is NULL");
    std::string n(name);
    if (n == "scan_unroll" && (value == 8 || value == 16)) x->opt_scan_unroll = value;
    else if (n == "queue_fronts" && value >= 0 && value <= 2) x->opt_queue_fronts = value;   // 0: by the size of the scan
    else if (n == "queue_min_mb" && value >= 0 && value <= (1 << 20)) x->opt_queue_min_mb = value;
    else if (n == "scan_split" && (value == 0 || value == 1 || value == 2 || value == 4)) x->opt_scan_split = value;   // 0: by block size
    else if (n == "scan_waves" && (value == 1 || value == 2 || value == 4 || value == 8)) x->opt_scan_waves = value;
    else if (n == "scan_prune" && value >= 0 && value <= 2) x->opt_scan_prune = value;   // 2 = also on small plans
    else if (n == "host_direct" && (value == 0 || value == 1)) {
        // 1: the scan kernel reads host-resident lists straight from pinned host memory
        // (no staging copies); 0: they are copied with hipMemcpyAsync on the side stream
        if (x->opt_host_direct != value) {
            if (moves_active(x)) return fail(IVF_ERR_INVALID, "host_direct cannot change while a budget change is in progress");
            x->opt_host_direct = value;
            if (x->ready) {
                HIP_TRY(hipDeviceSynchronize());
                int rc = upload_list_ptr_table(x);
                if (rc) return rc;
            }
        }
    }
    else if (n == "nside" && value >= 1 && value <= kMaxSide) x->opt_nside = value;
    else if (n == "residency_policy" && (value == 0 || value == 1)) x->opt_policy = value;   // 0 largest, 1 most probed
    else if (n == "segment_mb" && value >= 1 && value <= 65536) x->opt_segment_mb = value;  // next upload
    else if (n == "stage_mb" && value >= 1 && value <= 4096) x->opt_stage_mb = value;
    else if (n == "nstage" && value >= 2 && value <= kMaxStage) x->opt_nstage = value;
    // asynchronous budget changes: size of one batch of list copies, and how much may be under way at once
    else if (n == "regroup_fused" && (value == 0 || value == 1)) x->opt_regroup_fused = value;
    else if (n == "sel_threads" && (value == 0 || value == 256 || value == 1024)) x->opt_sel_threads = value;   // 0: by size
    else if (n == "move_chunk_kb" && value >= 1 && value <= ((int64_t)1 << 24)) x->opt_move_chunk_kb = value;
    else if (n == "move_inflight_kb" && value >= 1 && value <= ((int64_t)1 << 26)) x->opt_move_inflight_kb = value;
    else return fail(IVF_ERR_INVALID, "unknown option or bad value: %s=%lld", name, (long long)value);
    return 0;
}

}  // extern "C"
