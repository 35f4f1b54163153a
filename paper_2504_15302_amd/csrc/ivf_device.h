// Device-side building blocks shared by the kernels of the IVF retrieval path:
// order-preserving score keys and a workgroup-wide streaming top-k in LDS.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ivf {

constexpr int kLanes = 64;        // vectors per storage block = wavefront width
constexpr int kQB = 4;            // queries that share one read of a block
constexpr int kSelThreads = 1024; // workgroup size of the selection kernels (16 wavefronts:
                                  // the selection is latency-bound, it wants loads in flight)
constexpr int kChunk = 2048;      // keys sorted at a time by the streaming top-k
constexpr int kMaxK = 1024;       // largest k / nprobe
constexpr int kCoarseTile = 32;   // centroids per coarse tile maximum

// One unit of scan work: a block of 64 stored vectors against up to kQB queries.
struct ScanItem {
    const void* data;   // address of the block (HBM list arena or a staging buffer)
    uint32_t sblk;      // score block of the group's first query; query g adds g*nblk
    uint32_t nblk;      // blocks in the list
    uint16_t q[kQB];    // query rows of the group (entries past nq repeat the last one)
    uint16_t nq;        // queries in the group, 1..kQB
    uint16_t nvalid;    // valid vectors in the block, 1..64
    uint32_t shared;    // 1: other groups of queries read the same block (the list has more than kQB probes)
};
static_assert(sizeof(ScanItem) == 32, "ScanItem layout");

// Place of the item (group g of queries, block b) among the items of a list that `groups`
// groups of queries probe: the groups that read the same block are neighbours, so they run
// in the same or in neighbouring workgroups at about the same time and, reading with plain
// loads, find part of the block in the caches (what a nontemporal load brings in is not
// kept).  With one group the place is b.
__host__ __device__ inline unsigned item_slot(unsigned g, unsigned b, unsigned groups) {
    return b * groups + g;
}

// Monotone map float -> uint32 (larger score <=> larger key); -0 and +0 coincide.
__device__ __forceinline__ uint32_t ord_of(float s) {
    uint32_t u = __float_as_uint(s + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float score_of(uint32_t o) {
    return __uint_as_float((o & 0x80000000u) ? (o & 0x7fffffffu) : ~o);
}

// Sorts a[0..n) descending; n a power of two; all threads of the workgroup call it.
template <int T>
__device__ inline void bitonic_sort_desc(uint64_t* a, int n) {
    for (int size = 2; size <= n; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            for (int i = threadIdx.x; i < (n >> 1); i += T) {
                int lo = 2 * i - (i & (stride - 1));
                int hi = lo + stride;
                bool desc = ((lo & size) == 0) || (size == n);
                uint64_t x = a[lo], y = a[hi];
                if ((x < y) == desc) { a[lo] = y; a[hi] = x; }
            }
        }
    }
    __syncthreads();
}

// a[0..n) is bitonic; sorts it descending.
template <int T>
__device__ inline void bitonic_merge_desc(uint64_t* a, int n) {
    for (int stride = n >> 1; stride > 0; stride >>= 1) {
        __syncthreads();
        for (int i = threadIdx.x; i < (n >> 1); i += T) {
            int lo = 2 * i - (i & (stride - 1));
            int hi = lo + stride;
            uint64_t x = a[lo], y = a[hi];
            if (x < y) { a[lo] = y; a[hi] = x; }
        }
    }
    __syncthreads();
}

// Streaming top-k of unique 64-bit keys (0 = empty) kept sorted in LDS.
struct TopK {
    uint64_t top[kMaxK];
    uint64_t buf[kChunk];
    int count;   // keys waiting in buf
    int kp;      // power of two >= k
};

template <int T>
__device__ inline void topk_reset(TopK& t, int k) {
    int kp = 1;
    while (kp < k) kp <<= 1;
    for (int i = threadIdx.x; i < kp; i += T) t.top[i] = 0;
    if (threadIdx.x == 0) { t.count = 0; t.kp = kp; }
    __syncthreads();
}

// Merges the t.count keys waiting in buf into top.  Uniform call.  `finalize` maps a
// waiting key to its final form (e.g. replaces a handle in the low half by the
// tie-break rank) and runs once per key, all keys in parallel.
template <int T, class F>
__device__ inline void topk_flush(TopK& t, F finalize) {
    __syncthreads();
    const int m = t.count, kp = t.kp;
    if (m == 0) return;
    int n = kp;
    while (n < m) n <<= 1;
    for (int i = threadIdx.x; i < n; i += T) t.buf[i] = i < m ? finalize(t.buf[i]) : 0;
    bitonic_sort_desc<T>(t.buf, n);
    for (int i = threadIdx.x; i < kp; i += T) {
        uint64_t a = t.top[i], b = t.buf[kp - 1 - i];
        t.top[i] = a > b ? a : b;
    }
    bitonic_merge_desc<T>(t.top, kp);
    if (threadIdx.x == 0) t.count = 0;
    __syncthreads();
}

// Appends one key per calling lane that has `want` set; one LDS atomic per wavefront.
__device__ __forceinline__ void topk_append(TopK& t, bool want, uint64_t key) {
    uint64_t mask = __ballot(want);
    if (mask == 0) return;
    int lane = threadIdx.x & 63;
    int leader = __ffsll((long long)mask) - 1;
    int base = 0;
    if (lane == leader) base = atomicAdd(&t.count, __popcll(mask));
    base = __shfl(base, leader);
    if (want) {
        int off = __popcll(mask & ((1ull << lane) - 1ull));
        t.buf[base + off] = key;
    }
}

}  // namespace ivf
