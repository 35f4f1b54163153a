// Two-level exact k-selection, used twice: for the nprobe best centroid scores of a
// query and for the k best candidates among the scores of its probed lists.
//
// Values come in fixed-width blocks with a precomputed block maximum.  Level 1 finds
// the k-th largest block maximum M (a search on the order-preserving bits, four bits per
// round, no sorting): at least k values are >= M, so every member of the top-k is >= M and lives
// in a block whose maximum is >= M.  Level 2 visits only those blocks, keeps the values
// >= M (a few more than k unless scores tie massively) and sorts them with a streaming
// top-k in LDS, so any number of blocks and any number of ties is handled exactly.
// Keys are (order-preserving score bits, tie-break) and are unique per query, which
// makes the outcome independent of the order in which keys arrive.
#pragma once
#include "ivf_device.h"

namespace ivf {

constexpr int kOrdCache = 2 * kChunk;   // block maxima kept in LDS for the threshold search
                                        // (they borrow the top-k chunk buffer, idle in level 1)

struct SelectShared {
    TopK tk;
    int qual[kChunk];   // blocks that pass level 1
    int nqual;
    int wcount[2][kSelThreads / 64][16];   // per round parity and wavefront: counts for 15 candidate thresholds
};

// Src must provide:
//   int  nblocks() const
//   uint32_t block_max_ord(int f) const            order key of the block maximum
//   bool value(int f, int lane, uint32_t& ord, uint32_t& handle) const   per-lane value
//   uint32_t tiebreak(uint32_t handle) const       larger = preferred; unique per query
//   static constexpr int kWidth                    values per block (<= 64)
// `min_thr`: a lower bound of the k-th best value's order bits that the caller already
// knows (0 = none); blocks below it are not visited.
template <int T, class Src>
__device__ inline void two_level_select(SelectShared& sh, const Src& src, int k, uint32_t min_thr = 0) {
    const int nb = src.nblocks();
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    constexpr int kWaves = T / 64;
    constexpr int kPerWave = 64 / Src::kWidth;   // blocks a wavefront visits at once

    // level 1: thr = k-th largest block maximum (0 if there are fewer than k blocks),
    // i.e. the largest v such that at least k block maxima are >= v.
    uint32_t* ords = reinterpret_cast<uint32_t*>(sh.tk.buf);
    for (int i = threadIdx.x; i < min(nb, kOrdCache); i += T) ords[i] = src.block_max_ord(i);
    __syncthreads();
    auto ord_at = [&](int i) -> uint32_t { return i < kOrdCache ? ords[i] : src.block_max_ord(i); };
    // Four bits per round: every wavefront counts, for the 15 candidate values of the next
    // hex digit, how many of its block maxima reach the candidate; one barrier later the
    // first 15 lanes of every wavefront add up the wavefronts' counts and the digit is the
    // number of candidates that at least k maxima reach (the counts fall as the candidate
    // rises).  Eight barriers instead of one per bit: the workgroup is 16 wavefronts wide
    // and the barriers, not the counting, are what this search costs.
    uint32_t thr = 0;
    if (nb >= k) {
        for (int round = 0; round < 8; ++round) {
            const int shift = 28 - 4 * round;
            int cnt[15];
#pragma unroll
            for (int c = 0; c < 15; ++c) cnt[c] = 0;
            for (int i0 = 0; i0 < nb; i0 += T) {        // uniform trip count: ballots stay whole
                const int i = i0 + threadIdx.x;
                const bool in = i < nb;
                const uint32_t v = in ? ord_at(i) : 0u;
#pragma unroll
                for (int c = 0; c < 15; ++c)
                    cnt[c] += __popcll(__ballot(in && v >= (thr | ((uint32_t)(c + 1) << shift))));
            }
            const int slot = round & 1;
            int mine = 0;
#pragma unroll
            for (int c = 0; c < 15; ++c)
                if (lane == c) mine = cnt[c];
            if (lane < 15) sh.wcount[slot][wave][lane] = mine;
            __syncthreads();
            int total = 0;
            if (lane < 15) {
#pragma unroll
                for (int w = 0; w < kWaves; ++w) total += sh.wcount[slot][w][lane];
            }
            const unsigned long long reach = __ballot(lane < 15 && total >= k);
            thr |= (uint32_t)__popcll(reach) << shift;
        }
    }
    if (min_thr > thr) thr = min_thr;
    __syncthreads();     // the cached maxima are dead from here on: buf goes back to the top-k

    // level 2: values >= thr from blocks whose maximum is >= thr.  Survivors wait in
    // buf as (order bits, handle); their tie-breaks are looked up all at once at flush
    // time, so the dependent memory reads of a round overlap instead of queueing.
    auto finalize = [&](uint64_t key) -> uint64_t {
        return (key & 0xffffffff00000000ull) | src.tiebreak((uint32_t)key);
    };
    topk_reset<T>(sh.tk, k);
    for (int base = 0; base < nb; base += kChunk) {
        int m = min(kChunk, nb - base);
        if (threadIdx.x == 0) sh.nqual = 0;
        __syncthreads();
        for (int i = threadIdx.x; i < m; i += T) {
            // the cached maxima are still intact while nothing has been appended
            uint32_t o = base == 0 ? ord_at(i) : src.block_max_ord(base + i);
            if (o >= thr) sh.qual[atomicAdd(&sh.nqual, 1)] = base + i;
        }
        __syncthreads();
        const int nqual = sh.nqual;
        // rounds of at most 1024 appended keys, so buf (2048) cannot overflow
        constexpr int kRound = 1024 / 64 * kPerWave;         // blocks per round
        constexpr int kIter = (kRound + kWaves * kPerWave - 1) / (kWaves * kPerWave);
        for (int r0 = 0; r0 < nqual; r0 += kRound) {
            if (sh.tk.count > kChunk - 1024) topk_flush<T>(sh.tk, finalize);   // uniform: count read after a barrier
            uint32_t ordv[kIter], hv[kIter];
            bool okv[kIter];
#pragma unroll
            for (int it = 0; it < kIter; ++it) {
                int slot = (it * kWaves + wave) * kPerWave + lane / Src::kWidth;
                int idx = r0 + slot;
                okv[it] = slot < kRound && idx < nqual;
                ordv[it] = 0; hv[it] = 0;
                if (okv[it]) okv[it] = src.value(sh.qual[idx], lane % Src::kWidth, ordv[it], hv[it]);
            }
#pragma unroll
            for (int it = 0; it < kIter; ++it) {
                bool ok = okv[it] && ordv[it] >= thr;
                topk_append(sh.tk, ok, ((uint64_t)ordv[it] << 32) | hv[it]);
            }
            __syncthreads();
        }
    }
    topk_flush<T>(sh.tk, finalize);
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

// One workgroup per query: probes[q, 0..nprobe) = lists best first.  Also counts in
// hist[l] (zero on entry) how many queries probe list l (low 20 bits) and, above bit 20,
// for how many it is the best probe; of the latter only "non-zero" is used, as an
// ordering hint for the scan, so wrap-around there is harmless.
template <int T>
__global__ __launch_bounds__(T) void k_probe_select(const float* __restrict__ S,
                                                              const float* __restrict__ tmax,
                                                              int nlist, int ntile, int nprobe,
                                                              int32_t* __restrict__ probes,
                                                              int* __restrict__ hist) {
    __shared__ SelectShared sh;
    const int q = blockIdx.x;
    CoarseSrc src{S + (size_t)q * nlist, tmax + (size_t)q * ntile, nlist, ntile};
    two_level_select<T>(sh, src, nprobe);
    for (int i = threadIdx.x; i < nprobe; i += T) {
        uint64_t key = sh.tk.top[i];
        uint32_t lu = ~(uint32_t)key;               // nprobe <= nlist: never an empty key,
        int32_t l = lu < (uint32_t)nlist ? (int32_t)lu : 0;   // but stay in bounds on NaN input
        probes[(size_t)q * nprobe + i] = l;
        atomicAdd(&hist[l], 1 + (i == 0 ? (1 << 20) : 0));   // low 20 bits: probes; above: times best probe
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
template <int T>
__global__ __launch_bounds__(T) void k_final_select(
    const int32_t* __restrict__ probes, const uint32_t* __restrict__ pair_of_probe,
    const uint32_t* __restrict__ pair_start, const uint32_t* __restrict__ sblk_start, ListTable lt,
    const float* __restrict__ bmax, const float* __restrict__ scores,
    const uint32_t* __restrict__ rank_of_pos, const int64_t* __restrict__ id_sorted, int nprobe,
    int k, const unsigned long long* __restrict__ qthr, int64_t* __restrict__ out_ids,
    float* __restrict__ out_scores) {
    __shared__ SelectShared sh;
    __shared__ int pre[kMaxK + 1];
    __shared__ uint32_t sb[kMaxK];
    __shared__ int plen[kMaxK];
    __shared__ int64_t ppos0[kMaxK];
    const int q = blockIdx.x;
    for (int j = threadIdx.x; j < nprobe; j += T) {
        int l = probes[(size_t)q * nprobe + j];
        uint32_t p = pair_of_probe[(size_t)q * nprobe + j];
        int nb = lt.nblk[l];
        sb[j] = sblk_start[l] + (p - pair_start[l]) * (uint32_t)nb;
        plen[j] = lt.len[l];
        ppos0[j] = lt.pos0[l];
        pre[j + 1] = nb;
    }
    __syncthreads();
    if (threadIdx.x < 64) {       // prefix sums of the block counts by the first wavefront
        const int lane = threadIdx.x;
        int carry = 0;
        for (int j0 = 0; j0 < nprobe; j0 += 64) {
            int j = j0 + lane;
            int x = j < nprobe ? pre[j + 1] : 0;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                int y = __shfl_up(x, o);
                if (lane >= o) x += y;
            }
            if (j < nprobe) pre[j + 1] = carry + x;
            carry += __shfl(x, 63);
        }
        if (lane == 0) pre[0] = 0;
    }
    __syncthreads();
    ScanSrc src{pre, sb, plen, ppos0, nprobe, bmax, scores, rank_of_pos};
    // the scan stored a block's scores only if its maximum reached the bound it kept for
    // the query; the final bound is at least every bound it used, so visiting only blocks
    // at or above it never reads a block that was skipped
    two_level_select<T>(sh, src, k, qthr ? (uint32_t)qthr[q] : 0u);
    for (int i = threadIdx.x; i < k; i += T) {
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
