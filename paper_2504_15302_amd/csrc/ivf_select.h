// Two-level exact k-selection, used twice: for the nprobe best centroid scores of a
// query and for the k best candidates among the scores of its probed lists.
//
// Values come in fixed-width blocks with a precomputed block maximum.  Level 1 finds
// the k-th largest block maximum M: at least k values are >= M, so every member of
// the top-k is >= M and lives in a block whose maximum is >= M.  Level 2 visits only
// those blocks, keeps the values >= M and sorts them.  Both levels run on a streaming
// top-k in LDS, so any number of blocks and any number of ties is handled exactly.
// Keys are (order-preserving score bits, tie-break) and are unique per query, which
// makes the outcome independent of the order in which keys arrive.
#pragma once
#include "ivf_device.h"

namespace ivf {

struct SelectShared {
    TopK tk;
    int qual[kChunk];   // blocks that pass level 1
    int nqual;
    uint32_t thr;
};

// Src must provide:
//   int  nblocks() const
//   uint32_t block_max_ord(int f) const            order key of the block maximum
//   bool value(int f, int lane, uint32_t& ord, uint32_t& handle) const   per-lane value
//   uint32_t tiebreak(uint32_t handle) const       larger = preferred; unique per query
//   static constexpr int kWidth                    values per block (<= 64)
template <class Src>
__device__ inline void two_level_select(SelectShared& sh, const Src& src, int k) {
    constexpr int T = kSelThreads;
    const int nb = src.nblocks();
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    constexpr int kWaves = T / 64;
    constexpr int kPerWave = 64 / Src::kWidth;   // blocks a wavefront visits at once

    // level 1: k-th largest block maximum
    topk_reset<T>(sh.tk, k);
    for (int base = 0; base < nb; base += kChunk) {
        int m = min(kChunk, nb - base);
        for (int i = threadIdx.x; i < m; i += T)
            sh.tk.buf[i] = ((uint64_t)src.block_max_ord(base + i) << 32) | (uint32_t)(~(uint32_t)(base + i));
        if (threadIdx.x == 0) sh.tk.count = m;
        topk_flush<T>(sh.tk);
    }
    if (threadIdx.x == 0) sh.thr = (nb >= k) ? (uint32_t)(sh.tk.top[k - 1] >> 32) : 0u;
    __syncthreads();
    const uint32_t thr = sh.thr;

    // level 2: values >= thr from blocks whose maximum is >= thr
    topk_reset<T>(sh.tk, k);
    for (int base = 0; base < nb; base += kChunk) {
        int m = min(kChunk, nb - base);
        if (threadIdx.x == 0) sh.nqual = 0;
        __syncthreads();
        for (int i = threadIdx.x; i < m; i += T)
            if (src.block_max_ord(base + i) >= thr) sh.qual[atomicAdd(&sh.nqual, 1)] = base + i;
        __syncthreads();
        const int nqual = sh.nqual;
        // rounds of at most 1024 appended keys, so buf (2048) cannot overflow
        constexpr int kRound = 1024 / 64 * kPerWave;    // blocks per round
        for (int r0 = 0; r0 < nqual; r0 += kRound) {
            if (sh.tk.count > kChunk - 1024) topk_flush<T>(sh.tk);   // uniform: count read after a barrier
            for (int r = r0 + wave * kPerWave; r < min(nqual, r0 + kRound); r += kWaves * kPerWave) {
                int sub = lane / Src::kWidth;
                int idx = r + sub;
                bool ok = idx < nqual;
                uint32_t ord = 0, handle = 0;
                if (ok) ok = src.value(sh.qual[idx], lane % Src::kWidth, ord, handle) && ord >= thr;
                uint64_t key = 0;
                if (ok) key = ((uint64_t)ord << 32) | src.tiebreak(handle);
                topk_append(sh.tk, ok, key);
            }
            __syncthreads();
        }
    }
    topk_flush<T>(sh.tk);
}

// ---------------------------------------------------------------- probe selection
struct CoarseSrc {
    static constexpr int kWidth = kCoarseTile;
    const float* S;      // [nlist] scores of this query
    const float* tmax;   // [ntile]
    int nlist, ntile;
    __device__ int nblocks() const { return ntile; }
    __device__ uint32_t block_max_ord(int f) const { return ord_of(tmax[f]); }
    __device__ bool value(int f, int lane, uint32_t& ord, uint32_t& handle) const {
        int j = f * kCoarseTile + lane;
        if (j >= nlist) return false;
        ord = ord_of(S[j]);
        handle = (uint32_t)j;
        return true;
    }
    __device__ uint32_t tiebreak(uint32_t handle) const { return ~handle; }   // smaller list first
};

// One workgroup per query: probes[q, 0..nprobe) = lists best first; also counts how
// many queries probe each list (hist must be zero on entry).
__global__ __launch_bounds__(kSelThreads) void k_probe_select(const float* __restrict__ S,
                                                              const float* __restrict__ tmax,
                                                              int nlist, int ntile, int nprobe,
                                                              int32_t* __restrict__ probes,
                                                              int* __restrict__ hist) {
    __shared__ SelectShared sh;
    const int q = blockIdx.x;
    CoarseSrc src{S + (size_t)q * nlist, tmax + (size_t)q * ntile, nlist, ntile};
    two_level_select(sh, src, nprobe);
    for (int i = threadIdx.x; i < nprobe; i += kSelThreads) {
        uint64_t key = sh.tk.top[i];
        uint32_t lu = ~(uint32_t)key;               // nprobe <= nlist: never an empty key,
        int32_t l = lu < (uint32_t)nlist ? (int32_t)lu : 0;   // but stay in bounds on NaN input
        probes[(size_t)q * nprobe + i] = l;
        atomicAdd(&hist[l], 1);
    }
}

// ---------------------------------------------------------------- final selection
struct ListTable {
    const int32_t* len;      // [nlist] vectors per list
    const int32_t* nblk;     // [nlist] 64-vector blocks per list
    const int64_t* pos0;     // [nlist] upload position of the list's first vector
};

struct ScanSrc {
    static constexpr int kWidth = kLanes;
    // per-probe tables in LDS
    const int* pre;          // [nprobe+1] prefix of block counts
    const uint32_t* sb;      // [nprobe] first score block of the (query, list) pair
    const int* plen;         // [nprobe] list length
    const int64_t* ppos0;    // [nprobe] upload position of the list start
    int nprobe;
    const float* bmax;
    const float* scores;
    const uint32_t* rank_of_pos;
    __device__ int nblocks() const { return pre[nprobe]; }
    __device__ int probe_of(int f) const {
        int lo = 0, hi = nprobe;            // largest j with pre[j] <= f
        while (hi - lo > 1) {
            int mid = (lo + hi) >> 1;
            if (pre[mid] <= f) lo = mid; else hi = mid;
        }
        return lo;
    }
    __device__ uint32_t block_max_ord(int f) const {
        int j = probe_of(f);
        return ord_of(bmax[sb[j] + (uint32_t)(f - pre[j])]);
    }
    __device__ bool value(int f, int lane, uint32_t& ord, uint32_t& handle) const {
        int j = probe_of(f);
        int b = f - pre[j];
        int i = b * kLanes + lane;
        if (i >= plen[j]) return false;
        ord = ord_of(scores[(size_t)(sb[j] + (uint32_t)b) * kLanes + lane]);
        handle = (uint32_t)(ppos0[j] + i);
        return true;
    }
    __device__ uint32_t tiebreak(uint32_t handle) const { return ~rank_of_pos[handle]; }  // smaller id first
};

// One workgroup per query: the k best (score, id) over the scores the scan wrote.
__global__ __launch_bounds__(kSelThreads) void k_final_select(
    const int32_t* __restrict__ probes, const uint32_t* __restrict__ pair_of_probe,
    const uint32_t* __restrict__ pair_start, const uint32_t* __restrict__ sblk_start, ListTable lt,
    const float* __restrict__ bmax, const float* __restrict__ scores,
    const uint32_t* __restrict__ rank_of_pos, const int64_t* __restrict__ id_sorted, int nprobe,
    int k, int64_t* __restrict__ out_ids, float* __restrict__ out_scores) {
    __shared__ SelectShared sh;
    __shared__ int pre[kMaxK + 1];
    __shared__ uint32_t sb[kMaxK];
    __shared__ int plen[kMaxK];
    __shared__ int64_t ppos0[kMaxK];
    const int q = blockIdx.x;
    for (int j = threadIdx.x; j < nprobe; j += kSelThreads) {
        int l = probes[(size_t)q * nprobe + j];
        uint32_t p = pair_of_probe[(size_t)q * nprobe + j];
        int nb = lt.nblk[l];
        sb[j] = sblk_start[l] + (p - pair_start[l]) * (uint32_t)nb;
        plen[j] = lt.len[l];
        ppos0[j] = lt.pos0[l];
        pre[j + 1] = nb;
    }
    __syncthreads();
    if (threadIdx.x == 0) {       // nprobe <= 1024: a serial prefix is cheap next to the rest
        pre[0] = 0;
        for (int j = 0; j < nprobe; ++j) pre[j + 1] += pre[j];
    }
    __syncthreads();
    ScanSrc src{pre, sb, plen, ppos0, nprobe, bmax, scores, rank_of_pos};
    two_level_select(sh, src, k);
    for (int i = threadIdx.x; i < k; i += kSelThreads) {
        uint64_t key = sh.tk.top[i];
        int64_t id = -1;
        float s = -INFINITY;
        if (key != 0) {
            s = score_of((uint32_t)(key >> 32));
            id = id_sorted[~(uint32_t)key];
        }
        out_ids[(size_t)q * k + i] = id;
        out_scores[(size_t)q * k + i] = s;
    }
}

}  // namespace ivf
