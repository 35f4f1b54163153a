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

enum {                 // 64-bit counters accumulated by k_list_partial (zero on entry)
    kCntPairs = 0,
    kCntScoreBlocks = 1,
    kCntItems = 2,
    kCntUnique = 3,
    kCntVectors = 4,        // sum of len over probed lists
    kCntVectorsResident = 5,
    kNumCounters = 8
};

constexpr int kScanThreads = 1024;

// Exclusive prefix sums over the lists, two passes: each workgroup scans its 1024
// lists (one list per thread, coalesced) and publishes its totals; the second pass adds
// the totals of the workgroups before it.
__global__ __launch_bounds__(kScanThreads) void k_list_partial(
    const int* __restrict__ hist, const int32_t* __restrict__ nblk, const int32_t* __restrict__ len,
    const void* const* __restrict__ list_ptr, int nlist, uint32_t* __restrict__ pair_start,
    uint32_t* __restrict__ sblk_start, uint32_t* __restrict__ item_start,
    uint32_t* __restrict__ wg_totals, unsigned long long* __restrict__ counters) {
    __shared__ uint32_t wsum[kScanThreads / 64][3];
    __shared__ unsigned long long extra[3];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int l = blockIdx.x * kScanThreads + t;
    uint32_t v[3] = {0, 0, 0};
    unsigned long long uniq = 0, vec = 0, vres = 0;
    if (l < nlist) {
        unsigned cnt = (unsigned)hist[l];
        if (cnt) {
            unsigned nb = (unsigned)nblk[l];
            bool res = list_ptr[l] != nullptr;
            v[0] = cnt;
            v[1] = cnt * nb;
            v[2] = res ? nb * ((cnt + kQB - 1) / kQB) : 0;
            uniq = 1;
            vec = (unsigned)len[l];
            vres = res ? vec : 0;
        }
    }
    if (t == 0) extra[0] = extra[1] = extra[2] = 0;
    uint32_t inc[3];
#pragma unroll
    for (int c = 0; c < 3; ++c) {           // inclusive scan inside the wavefront
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
    uint32_t base[3] = {0, 0, 0}, total[3] = {0, 0, 0};
    for (int w = 0; w < kScanThreads / 64; ++w)
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            uint32_t x = wsum[w][c];
            if (w < wave) base[c] += x;
            total[c] += x;
        }
    if (l < nlist) {
        pair_start[l] = base[0] + inc[0] - v[0];
        sblk_start[l] = base[1] + inc[1] - v[1];
        item_start[l] = base[2] + inc[2] - v[2];
    }
    __syncthreads();
    if (t == 0) {
#pragma unroll
        for (int c = 0; c < 3; ++c) wg_totals[blockIdx.x * 3 + c] = total[c];
        atomicAdd(&counters[kCntPairs], (unsigned long long)total[0]);
        atomicAdd(&counters[kCntScoreBlocks], (unsigned long long)total[1]);
        atomicAdd(&counters[kCntItems], (unsigned long long)total[2]);
        atomicAdd(&counters[kCntUnique], extra[0]);
        atomicAdd(&counters[kCntVectors], extra[1]);
        atomicAdd(&counters[kCntVectorsResident], extra[2]);
    }
}

__global__ __launch_bounds__(kScanThreads) void k_list_finish(
    int nlist, const uint32_t* __restrict__ wg_totals, uint32_t* __restrict__ pair_start,
    uint32_t* __restrict__ sblk_start, uint32_t* __restrict__ item_start) {
    __shared__ uint32_t red[kScanThreads / 64][3];
    __shared__ uint32_t base[3];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    uint32_t s[3] = {0, 0, 0};
    for (int w = t; w < (int)blockIdx.x; w += kScanThreads)
#pragma unroll
        for (int c = 0; c < 3; ++c) s[c] += wg_totals[w * 3 + c];
#pragma unroll
    for (int c = 0; c < 3; ++c) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) s[c] += __shfl_xor(s[c], o);
        if (lane == 0) red[wave][c] = s[c];
    }
    __syncthreads();
    if (t < 3) {
        uint32_t x = 0;
        for (int w = 0; w < kScanThreads / 64; ++w) x += red[w][t];
        base[t] = x;
    }
    __syncthreads();
    const int l = blockIdx.x * kScanThreads + t;
    if (l < nlist && blockIdx.x > 0) {
        pair_start[l] += base[0];
        sblk_start[l] += base[1];
        item_start[l] += base[2];
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
