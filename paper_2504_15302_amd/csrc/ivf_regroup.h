// Regrouping of the (query, probed list) pairs by list, entirely on the device, so
// that each probed list is read once for all the queries that probe it, and the
// work plan of the scan (one item per 64-vector block and group of up to kQB queries).
//
// Numbering (the host mirrors it when lists have to be streamed from host memory):
//   pairs are ordered by (list ascending, query ascending);
//   pair_start[l]  = number of pairs of lists < l
//   sblk_start[l]  = sum over lists l' < l of cnt[l'] * nblk[l']   (score blocks)
//   item_start[l]  = sum over HBM-resident lists l' < l of nblk[l'] * ceil(cnt[l']/kQB)
#pragma once
#include "ivf_device.h"

namespace ivf {

enum {                 // 64-bit counters accumulated by k_list_partial (zero on entry)
    kCntPairs = 0,
    kCntScoreBlocks = 1,
    kCntItems = 2,
    kCntUnique = 3,
    kCntVectors = 4,        // sum of len over probed lists
    kCntVectorsResident = 5,
    kNumCounters = 8
};

constexpr int kScanThreads = 1024;   // lists per workgroup of the prefix kernels when they have the GPU to themselves
constexpr int kScanThreadsShared = 256;   // ... and under another search's scan: a workgroup of sixteen wavefronts finds
                                          // no room on a compute unit until the scan's grid has drained, one of four does
constexpr int kHistTopShift = 20;                         // hist[l] = probes + (times best probe << 20)
constexpr int kHistCountMask = (1 << kHistTopShift) - 1;
constexpr int kScanVals = 4;   // pairs, score blocks, items of "first" lists, items of the other lists

// Exclusive prefix sums over the lists, two passes: each workgroup scans its 1024
// lists (one list per thread, coalesced) and publishes its totals; the second pass adds
// the totals of the workgroups before it.  Scan items are numbered in two classes: lists
// that are some query's best probe come first, so that the scan meets every query's most
// promising list early and its bound on the k-th best score is tight almost from the start.
template <int T>
__global__ __launch_bounds__(T) void k_list_partial(
    const int* __restrict__ hist, const int32_t* __restrict__ nblk, const int32_t* __restrict__ len,
    const void* const* __restrict__ list_ptr, int nlist, uint32_t* __restrict__ pair_start,
    uint32_t* __restrict__ sblk_start, uint32_t* __restrict__ item_start,
    uint32_t* __restrict__ wg_totals, unsigned long long* __restrict__ counters) {
    __shared__ uint32_t wsum[T / 64][kScanVals];
    __shared__ unsigned long long extra[3];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int l = blockIdx.x * T + t;
    uint32_t v[kScanVals] = {0, 0, 0, 0};
    unsigned long long uniq = 0, vec = 0, vres = 0;
    bool first = false;
    if (l < nlist) {
        const unsigned h = (unsigned)hist[l];
        const unsigned cnt = h & kHistCountMask;
        if (cnt) {
            unsigned nb = (unsigned)nblk[l];
            const uintptr_t lp = reinterpret_cast<uintptr_t>(list_ptr[l]);
            bool res = lp != 0;                      // readable by the scan kernel
            const bool in_hbm = res && !(lp & 1u);   // bit 0 tags a pinned-host address
            first = (h >> kHistTopShift) != 0;
            v[0] = cnt;
            v[1] = cnt * nb;
            unsigned items = res ? nb * ((cnt + kQB - 1) / kQB) : 0;
            v[first ? 2 : 3] = items;
            uniq = 1;
            vec = (unsigned)len[l];
            vres = in_hbm ? vec : 0;
        }
    }
    if (t == 0) extra[0] = extra[1] = extra[2] = 0;
    uint32_t inc[kScanVals];
#pragma unroll
    for (int c = 0; c < kScanVals; ++c) {           // inclusive scan inside the wavefront
        uint32_t x = v[c];
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            uint32_t y = __shfl_up(x, o);
            if (lane >= o) x += y;
        }
        inc[c] = x;
        if (lane == 63) wsum[wave][c] = x;
    }
    __syncthreads();
    if (uniq) {
        atomicAdd(&extra[0], uniq);
        atomicAdd(&extra[1], vec);
        atomicAdd(&extra[2], vres);
    }
    uint32_t base[kScanVals] = {0, 0, 0, 0}, total[kScanVals] = {0, 0, 0, 0};
    for (int w = 0; w < T / 64; ++w)
#pragma unroll
        for (int c = 0; c < kScanVals; ++c) {
            uint32_t x = wsum[w][c];
            if (w < wave) base[c] += x;
            total[c] += x;
        }
    if (l < nlist) {
        pair_start[l] = base[0] + inc[0] - v[0];
        sblk_start[l] = base[1] + inc[1] - v[1];
        item_start[l] = first ? base[2] + inc[2] - v[2] : base[3] + inc[3] - v[3];   // within its class
    }
    __syncthreads();
    if (t == 0) {
#pragma unroll
        for (int c = 0; c < kScanVals; ++c) wg_totals[blockIdx.x * kScanVals + c] = total[c];
        atomicAdd(&counters[kCntPairs], (unsigned long long)total[0]);
        atomicAdd(&counters[kCntScoreBlocks], (unsigned long long)total[1]);
        atomicAdd(&counters[kCntItems], (unsigned long long)total[2] + total[3]);
        atomicAdd(&counters[kCntUnique], extra[0]);
        atomicAdd(&counters[kCntVectors], extra[1]);
        atomicAdd(&counters[kCntVectorsResident], extra[2]);
    }
}

template <int T>
__global__ __launch_bounds__(T) void k_list_finish(
    const int* __restrict__ hist, int nlist, int nwg, const uint32_t* __restrict__ wg_totals,
    uint32_t* __restrict__ pair_start, uint32_t* __restrict__ sblk_start,
    uint32_t* __restrict__ item_start) {
    __shared__ uint32_t red[T / 64][kScanVals + 1];
    __shared__ uint32_t base[kScanVals + 1];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    uint32_t s[kScanVals + 1] = {0, 0, 0, 0, 0};      // [4] = items of "first" lists, all workgroups
    for (int w = t; w < nwg; w += T) {
        if (w < (int)blockIdx.x)
#pragma unroll
            for (int c = 0; c < kScanVals; ++c) s[c] += wg_totals[w * kScanVals + c];
        s[kScanVals] += wg_totals[w * kScanVals + 2];
    }
#pragma unroll
    for (int c = 0; c <= kScanVals; ++c) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) s[c] += __shfl_xor(s[c], o);
        if (lane == 0) red[wave][c] = s[c];
    }
    __syncthreads();
    if (t <= kScanVals) {
        uint32_t x = 0;
        for (int w = 0; w < T / 64; ++w) x += red[w][t];
        base[t] = x;
    }
    __syncthreads();
    const int l = blockIdx.x * T + t;
    if (l < nlist) {
        const bool first = ((unsigned)hist[l] >> kHistTopShift) != 0;
        pair_start[l] += base[0];
        sblk_start[l] += base[1];
        item_start[l] += first ? base[2] : base[kScanVals] + base[3];
    }
}

// One thread per (query, probe): drops the pair into its list's segment.
__global__ void k_pair_fill(const int32_t* __restrict__ probes, int npairs,
                            const uint32_t* __restrict__ pair_start, int* __restrict__ cursor,
                            uint32_t* __restrict__ pair_flat) {
    int f = blockIdx.x * blockDim.x + threadIdx.x;
    if (f >= npairs) return;
    int l = probes[f];
    int slot = atomicAdd(&cursor[l], 1);
    pair_flat[pair_start[l] + slot] = (uint32_t)f;
}

// One thread per list: orders its segment by query, fills the pair tables and writes
// the scan items of the list if it is HBM-resident.
__global__ void k_plan(const int* __restrict__ hist, const int32_t* __restrict__ nblk,
                       const int32_t* __restrict__ len, const void* const* __restrict__ list_ptr,
                       int nlist, int nprobe, size_t block_bytes,
                       const uint32_t* __restrict__ pair_start,
                       const uint32_t* __restrict__ sblk_start,
                       const uint32_t* __restrict__ item_start, uint32_t* __restrict__ pair_flat,
                       uint32_t* __restrict__ pair_of_probe, ScanItem* __restrict__ items,
                       uint32_t* __restrict__ hits) {
    int l = blockIdx.x * blockDim.x + threadIdx.x;
    if (l >= nlist) return;
    const unsigned cnt = (unsigned)hist[l] & kHistCountMask;
    if (!cnt) return;
    atomicAdd(&hits[l], cnt);        // lifetime probe count of the list (residency policy); queued searches may regroup side by side
    const uint32_t ps = pair_start[l];
    uint32_t* seg = pair_flat + ps;
    for (unsigned i = 1; i < cnt; ++i) {        // insertion sort: segments are tiny
        uint32_t v = seg[i];
        int j = (int)i - 1;
        while (j >= 0 && seg[j] > v) { seg[j + 1] = seg[j]; --j; }
        seg[j + 1] = v;
    }
    for (unsigned i = 0; i < cnt; ++i) {
        pair_of_probe[seg[i]] = ps + i;
    }
    const char* base = reinterpret_cast<const char*>(reinterpret_cast<uintptr_t>(list_ptr[l]) & ~(uintptr_t)1);
    if (!base) return;
    const unsigned nb = (unsigned)nblk[l];
    const unsigned ln = (unsigned)len[l];
    const unsigned groups = (cnt + kQB - 1) / kQB;
    ScanItem* out = items + item_start[l];
    for (unsigned g = 0; g < groups; ++g) {
        unsigned nqg = min((unsigned)kQB, cnt - g * kQB);
        for (unsigned b = 0; b < nb; ++b) {
            ScanItem it;
            it.data = base + (size_t)b * block_bytes;
            it.sblk = sblk_start[l] + g * kQB * nb + b;
            it.nblk = nb;
#pragma unroll
            for (unsigned j = 0; j < kQB; ++j)
                it.q[j] = (uint16_t)(seg[g * kQB + min(j, nqg - 1)] / (uint32_t)nprobe);
            it.nq = (uint16_t)nqg;
            it.nvalid = (uint16_t)min(64u, ln - b * 64u);
            it.shared = groups > 1 ? 1u : 0u;
            out[item_slot(g, b, groups)] = it;
        }
    }
}


// The whole regrouping in one workgroup, for searches whose lists and pairs are few enough
// that four launches cost more than the work: the same numbering as k_list_partial /
// k_list_finish, the same segments as k_pair_fill, the same items as k_plan, with
// workgroup barriers where the separate kernels have launch boundaries.
constexpr int kFusedMaxLists = 1024, kFusedMaxPairs = 2048;
template <int T>
__global__ __launch_bounds__(T) void k_regroup_small(
    const int* __restrict__ hist, const int32_t* __restrict__ nblk, const int32_t* __restrict__ len,
    const void* const* __restrict__ list_ptr, int nlist, int nprobe, size_t block_bytes,
    const int32_t* __restrict__ probes, int npairs, int* __restrict__ cursor,
    uint32_t* __restrict__ pair_start, uint32_t* __restrict__ sblk_start, uint32_t* __restrict__ item_start,
    uint32_t* __restrict__ pair_flat, uint32_t* __restrict__ pair_of_probe, ScanItem* __restrict__ items,
    uint32_t* __restrict__ hits, unsigned long long* __restrict__ counters) {
    __shared__ uint32_t wsum[T / 64][kScanVals];
    __shared__ uint32_t run[kScanVals];              // totals of the chunks done so far
    __shared__ unsigned long long extra[3];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    if (t < kScanVals) run[t] = 0;
    if (t < 3) extra[t] = 0;
    __syncthreads();
    // 1. exclusive prefix sums over the lists (the loop runs once for up to 1024 lists)
    for (int c0 = 0; c0 < nlist; c0 += T) {
        const int l = c0 + t;
        uint32_t v[kScanVals] = {0, 0, 0, 0};
        unsigned long long uniq = 0, vec = 0, vres = 0;
        bool first = false;
        if (l < nlist) {
            const unsigned h = (unsigned)hist[l];
            const unsigned cnt = h & kHistCountMask;
            if (cnt) {
                const unsigned nb = (unsigned)nblk[l];
                const uintptr_t lp = reinterpret_cast<uintptr_t>(list_ptr[l]);
                const bool res = lp != 0, in_hbm = res && !(lp & 1u);
                first = (h >> kHistTopShift) != 0;
                v[0] = cnt;
                v[1] = cnt * nb;
                v[first ? 2 : 3] = res ? nb * ((cnt + kQB - 1) / kQB) : 0;
                uniq = 1;
                vec = (unsigned)len[l];
                vres = in_hbm ? vec : 0;
            }
        }
        uint32_t inc[kScanVals];
#pragma unroll
        for (int c = 0; c < kScanVals; ++c) {
            uint32_t x = v[c];
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                uint32_t y = __shfl_up(x, o);
                if (lane >= o) x += y;
            }
            inc[c] = x;
            if (lane == 63) wsum[wave][c] = x;
        }
        if (uniq) {
            atomicAdd(&extra[0], uniq);
            atomicAdd(&extra[1], vec);
            atomicAdd(&extra[2], vres);
        }
        __syncthreads();
        uint32_t base[kScanVals], total[kScanVals];
#pragma unroll
        for (int c = 0; c < kScanVals; ++c) { base[c] = run[c]; total[c] = 0; }
        for (int w = 0; w < T / 64; ++w)
#pragma unroll
            for (int c = 0; c < kScanVals; ++c) {
                uint32_t x = wsum[w][c];
                if (w < wave) base[c] += x;
                total[c] += x;
            }
        if (l < nlist) {
            pair_start[l] = base[0] + inc[0] - v[0];
            sblk_start[l] = base[1] + inc[1] - v[1];
            item_start[l] = first ? base[2] + inc[2] - v[2] : base[3] + inc[3] - v[3];   // within its class
        }
        __syncthreads();
        if (t < kScanVals) run[t] += total[t];
        __syncthreads();
    }
    if (t == 0) {
        counters[kCntPairs] = run[0];
        counters[kCntScoreBlocks] = run[1];
        counters[kCntItems] = (unsigned long long)run[2] + run[3];
        counters[kCntUnique] = extra[0];
        counters[kCntVectors] = extra[1];
        counters[kCntVectorsResident] = extra[2];
    }
    const uint32_t first_items = run[2];             // items of the other lists come after these
    // 2. every (query, probe) pair drops into its list's segment
    for (int f = t; f < npairs; f += T) {
        const int l = probes[f];
        const int slot = atomicAdd(&cursor[l], 1);
        pair_flat[pair_start[l] + slot] = (uint32_t)f;
    }
    __syncthreads();
    // 3. per list: order the segment by query, fill the pair table, write the scan items
    for (int l = t; l < nlist; l += T) {
        const unsigned h = (unsigned)hist[l];
        const unsigned cnt = h & kHistCountMask;
        if (!cnt) continue;
        atomicAdd(&hits[l], cnt);
        const uint32_t ps = pair_start[l];
        uint32_t* seg = pair_flat + ps;
        for (unsigned i = 1; i < cnt; ++i) {
            uint32_t v = seg[i];
            int j = (int)i - 1;
            while (j >= 0 && seg[j] > v) { seg[j + 1] = seg[j]; --j; }
            seg[j + 1] = v;
        }
        for (unsigned i = 0; i < cnt; ++i) pair_of_probe[seg[i]] = ps + i;
        const char* base = reinterpret_cast<const char*>(reinterpret_cast<uintptr_t>(list_ptr[l]) & ~(uintptr_t)1);
        if (!base) continue;
        const unsigned nb = (unsigned)nblk[l];
        const unsigned ln = (unsigned)len[l];
        const unsigned groups = (cnt + kQB - 1) / kQB;
        const uint32_t is = item_start[l] + ((h >> kHistTopShift) != 0 ? 0u : first_items);
        ScanItem* out = items + is;
        for (unsigned g = 0; g < groups; ++g) {
            const unsigned nqg = min((unsigned)kQB, cnt - g * kQB);
            for (unsigned b = 0; b < nb; ++b) {
                ScanItem it;
                it.data = base + (size_t)b * block_bytes;
                it.sblk = sblk_start[l] + g * kQB * nb + b;
                it.nblk = nb;
#pragma unroll
                for (unsigned j = 0; j < kQB; ++j)
                    it.q[j] = (uint16_t)(seg[g * kQB + min(j, nqg - 1)] / (uint32_t)nprobe);
                it.nq = (uint16_t)nqg;
                it.nvalid = (uint16_t)min(64u, ln - b * 64u);
                it.shared = groups > 1 ? 1u : 0u;
                out[item_slot(g, b, groups)] = it;
            }
        }
    }
}

}  // namespace ivf
