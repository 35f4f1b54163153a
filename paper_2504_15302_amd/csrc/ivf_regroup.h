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

__global__ void k_zero_i32(int* __restrict__ p, size_t n) {
    size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

enum {                 // 64-bit counters written by k_list_scan
    kCntPairs = 0,
    kCntScoreBlocks = 1,
    kCntItems = 2,
    kCntUnique = 3,
    kCntVectors = 4,        // sum of len over probed lists
    kCntVectorsResident = 5,
    kNumCounters = 8
};

constexpr int kScanThreads = 1024;

// Single workgroup: exclusive prefix sums over the lists.
__global__ __launch_bounds__(kScanThreads) void k_list_scan(
    const int* __restrict__ hist, const int32_t* __restrict__ nblk, const int32_t* __restrict__ len,
    const void* const* __restrict__ list_ptr, int nlist, uint32_t* __restrict__ pair_start,
    uint32_t* __restrict__ sblk_start, uint32_t* __restrict__ item_start,
    unsigned long long* __restrict__ counters) {
    __shared__ unsigned long long part[kScanThreads][3];
    __shared__ unsigned long long extra[3];
    const int t = threadIdx.x;
    const int per = (nlist + kScanThreads - 1) / kScanThreads;
    const int l0 = min(nlist, t * per), l1 = min(nlist, l0 + per);
    unsigned long long a = 0, b = 0, c = 0, uniq = 0, vec = 0, vres = 0;
    for (int l = l0; l < l1; ++l) {
        unsigned cnt = (unsigned)hist[l];
        if (cnt) {
            unsigned nb = (unsigned)nblk[l];
            bool res = list_ptr[l] != nullptr;
            a += cnt;
            b += (unsigned long long)cnt * nb;
            if (res) c += (unsigned long long)nb * ((cnt + kQB - 1) / kQB);
            uniq += 1;
            vec += (unsigned)len[l];
            if (res) vres += (unsigned)len[l];
        }
    }
    part[t][0] = a; part[t][1] = b; part[t][2] = c;
    if (t == 0) extra[0] = extra[1] = extra[2] = 0;
    __syncthreads();
    atomicAdd(&extra[0], uniq);
    atomicAdd(&extra[1], vec);
    atomicAdd(&extra[2], vres);
    // inclusive Hillis-Steele scan over the per-thread sums
    for (int off = 1; off < kScanThreads; off <<= 1) {
        unsigned long long x0 = 0, x1 = 0, x2 = 0;
        if (t >= off) { x0 = part[t - off][0]; x1 = part[t - off][1]; x2 = part[t - off][2]; }
        __syncthreads();
        part[t][0] += x0; part[t][1] += x1; part[t][2] += x2;
        __syncthreads();
    }
    unsigned long long ea = part[t][0] - a, eb = part[t][1] - b, ec = part[t][2] - c;
    for (int l = l0; l < l1; ++l) {
        pair_start[l] = (uint32_t)ea;
        sblk_start[l] = (uint32_t)eb;
        item_start[l] = (uint32_t)ec;
        unsigned cnt = (unsigned)hist[l];
        if (cnt) {
            unsigned nb = (unsigned)nblk[l];
            ea += cnt;
            eb += (unsigned long long)cnt * nb;
            if (list_ptr[l] != nullptr) ec += (unsigned long long)nb * ((cnt + kQB - 1) / kQB);
        }
    }
    if (t == kScanThreads - 1) {
        counters[kCntPairs] = part[t][0];
        counters[kCntScoreBlocks] = part[t][1];
        counters[kCntItems] = part[t][2];
        counters[kCntUnique] = extra[0];
        counters[kCntVectors] = extra[1];
        counters[kCntVectorsResident] = extra[2];
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
                       uint32_t* __restrict__ pair_q, uint32_t* __restrict__ pair_of_probe,
                       ScanItem* __restrict__ items) {
    int l = blockIdx.x * blockDim.x + threadIdx.x;
    if (l >= nlist) return;
    const unsigned cnt = (unsigned)hist[l];
    if (!cnt) return;
    const uint32_t ps = pair_start[l];
    uint32_t* seg = pair_flat + ps;
    for (unsigned i = 1; i < cnt; ++i) {        // insertion sort: segments are tiny
        uint32_t v = seg[i];
        int j = (int)i - 1;
        while (j >= 0 && seg[j] > v) { seg[j + 1] = seg[j]; --j; }
        seg[j + 1] = v;
    }
    for (unsigned i = 0; i < cnt; ++i) {
        uint32_t f = seg[i];
        pair_q[ps + i] = f / (uint32_t)nprobe;
        pair_of_probe[f] = ps + i;
    }
    const char* base = static_cast<const char*>(list_ptr[l]);
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
            it.pair0 = ps + g * kQB;
            it.nq = nqg;
            it.nvalid = min(64u, ln - b * 64u);
            it.pad = 0;
            out[g * nb + b] = it;
        }
    }
}

}  // namespace ivf
