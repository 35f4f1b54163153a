// The list scan: inner products of every vector of every probed list with every query
// that probes the list.  HBM-bound (about one multiply-add per byte loaded), so the
// kernel is built around the loads:
//   * storage is blocked as [block of 64 vectors][d/E chunks][64 lanes][16 bytes]
//     (E = 8 for fp16, 4 for fp32, 16 for int8 codes): a lane owns one vector, every
//     load instruction of a wavefront fetches one contiguous 1 KiB line, and no
//     cross-lane reduction is needed for the dot product; int8 blocks end with the 64
//     fp32 scales of their vectors (the stored vector is scale * codes);
//   * a wavefront streams one block (64*d*elem bytes, contiguous) with two register
//     buffers of U loads each, so loads of the next chunk group are in flight while
//     the current one is multiplied;
//   * the query values are wave-uniform: a lane loads one query value per dimension of
//     the group (one coalesced load per query and group, served by L2), and each value
//     is broadcast with a lane read and enters the FMA as a scalar operand — no LDS,
//     no dependence on d, one vector register per query and 64 dimensions;
//   * up to kQB queries that probe the same list share one read of the block;
//   * the maximum of each block of 64 scores always goes to a scratch array; the 64
//     scores themselves (4 bytes per vector and query, ~0.3 % of the bytes read — but
//     measured to cost ~5 % of the read bandwidth when all are stored) are stored only
//     for blocks whose maximum reaches a running lower bound of the query's k-th best
//     score.  The final selection visits only blocks at or above the final bound, so it
//     never reads a block that was skipped.
#pragma once
#include "ivf_device.h"

namespace ivf {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));
typedef const u4 __attribute__((address_space(1))) * gptr_u4;   // global (HBM) address space

// max over the 64 lanes through the LDS crossbar (no LDS memory is touched)
__device__ __forceinline__ float wave_max(float v, int lane) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        int other = __builtin_amdgcn_ds_bpermute((lane ^ o) << 2, __float_as_int(v));
        v = fmaxf(v, __int_as_float(other));
    }
    return v;
}

// storage types (the dtype codes of the C ABI)
constexpr int kF32 = 0, kF16 = 1, kI8 = 2;
template <int ST> struct Store;
template <> struct Store<kF32> { static constexpr int E = 4; };
template <> struct Store<kF16> { static constexpr int E = 8; };
template <> struct Store<kI8> { static constexpr int E = 16; };

// One group of UU consecutive 16-byte chunks of the lane's vector plus the matching
// slice of each query, spread one value per lane (lane j holds dimension dim0 + j).
template <int NQ, int UU, int E>
struct ScanBuf {
    static constexpr int G = UU * E;             // dimensions covered
    static constexpr int QV = (G + 63) / 64;     // query registers per query
    u4 x[UU];
    float q[NQ][QV];
};

// KEEP: plain loads, so that the block stays in L2 for the other query groups that read
// it; otherwise nontemporal loads (worth 10 % to a scan that reads everything once).
template <bool KEEP, int NQ, int UU, int E>
__device__ __forceinline__ void load_group(ScanBuf<NQ, UU, E>& b, gptr_u4 src, int chunk0,
                                           const float* const (&qrow)[NQ], int lane) {
    using B = ScanBuf<NQ, UU, E>;
#pragma unroll
    for (int u = 0; u < UU; ++u) {
        if (KEEP) b.x[u] = src[(size_t)(chunk0 + u) * kLanes];
        else b.x[u] = __builtin_nontemporal_load(src + (size_t)(chunk0 + u) * kLanes);
    }
    const int dim0 = chunk0 * E;
#pragma unroll
    for (int g = 0; g < NQ; ++g)
#pragma unroll
        for (int v = 0; v < B::QV; ++v) {
            int j = v * 64 + lane;
            if (B::G % 64 != 0) j = min(j, B::G - 1);     // idle lanes re-read the last value
            b.q[g][v] = qrow[g][dim0 + j];
        }
}

// acc[g] += sum over the group's dimensions of x * q[g]; the query value of a
// dimension is broadcast from the lane that holds it and enters the FMA as a scalar.
// Eight dimensions at a time (half a chunk of int8 codes), so that the broadcast values
// of one step fit the scalar registers.
template <int ST, int NQ, int UU, int E>
__device__ __forceinline__ void fma_group(const ScanBuf<NQ, UU, E>& b, float (&acc)[NQ]) {
    constexpr int S = E < 8 ? E : 8;             // dimensions per step
#pragma unroll
    for (int u = 0; u < UU; ++u) {
#pragma unroll
        for (int h0 = 0; h0 < E; h0 += S) {
            float xf[S];
            if constexpr (ST == kF16) {
                h8 x = __builtin_bit_cast(h8, b.x[u]);
#pragma unroll
                for (int h = 0; h < S; ++h) xf[h] = (float)x[h];
            } else if constexpr (ST == kF32) {
                f4 x = __builtin_bit_cast(f4, b.x[u]);
#pragma unroll
                for (int h = 0; h < S; ++h) xf[h] = x[h];
            } else {
#pragma unroll
                for (int h = 0; h < S; ++h) {
                    const unsigned w = b.x[u][(h0 + h) / 4];
                    xf[h] = (float)(int)(signed char)(w >> (8 * ((h0 + h) % 4)));
                }
            }
            // The empty asm makes the query register opaque here, so the lane reads of this
            // step stay next to its FMAs; hoisted to the load they would need 64 scalar
            // registers per query and spill.
            float qreg[NQ];
#pragma unroll
            for (int g = 0; g < NQ; ++g) {
                qreg[g] = b.q[g][(u * E + h0) / 64];
                asm volatile("" : "+v"(qreg[g]));
            }
            float qs[NQ][S];
#pragma unroll
            for (int h = 0; h < S; ++h)
#pragma unroll
                for (int g = 0; g < NQ; ++g)
                    qs[g][h] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(qreg[g]), (u * E + h0 + h) % 64));
#pragma unroll
            for (int h = 0; h < S; ++h)
#pragma unroll
                for (int g = 0; g < NQ; ++g) acc[g] = __builtin_fmaf(xf[h], qs[g][h], acc[g]);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// Inner products of the lane's vector with the NQ queries of the item over the 16-byte
// chunks [c0, c1) of the vector: acc[g] = sum in ascending chunk order, starting from 0.
template <int ST, int NQ, int U, bool KEEP = false>
__device__ __forceinline__ void scan_accumulate(const ScanItem& it, const float* __restrict__ Q, int d,
                                                int c0, int c1, int lane, float (&acc)[kQB]) {
    constexpr int E = Store<ST>::E;
    // lanes past the end of the list re-read the last valid vector (same cache lines,
    // no extra traffic, no divergence); their results are discarded later
    const int ld_lane = min(lane, (int)it.nvalid - 1);
    const gptr_u4 src = (gptr_u4)(uintptr_t)it.data + ld_lane;

    const float* qrow[NQ];
#pragma unroll
    for (int g = 0; g < NQ; ++g) {
        qrow[g] = Q + (size_t)it.q[g] * d;
    }
    float a[NQ];
#pragma unroll
    for (int g = 0; g < NQ; ++g) a[g] = 0.f;

    // two register buffers: the loads of group i+1 are in flight while group i is used
    ScanBuf<NQ, U, E> bufA, bufB;
    const int ngroup = (c1 - c0) / U;
    if (ngroup > 0) {
        int gi = 0;
        load_group<KEEP>(bufA, src, c0, qrow, lane);
        for (; gi + 2 < ngroup; gi += 2) {           // bufA holds group gi
            load_group<KEEP>(bufB, src, c0 + (gi + 1) * U, qrow, lane);
            fma_group<ST>(bufA, a);
            load_group<KEEP>(bufA, src, c0 + (gi + 2) * U, qrow, lane);
            fma_group<ST>(bufB, a);
        }
        if (gi + 1 < ngroup) {
            load_group<KEEP>(bufB, src, c0 + (gi + 1) * U, qrow, lane);
            fma_group<ST>(bufA, a);
            fma_group<ST>(bufB, a);
        } else {
            fma_group<ST>(bufA, a);
        }
    }
    for (int c = c0 + ngroup * U; c < c1; ++c) {    // the range is not a multiple of the group width
        ScanBuf<NQ, 1, E> one;
        load_group<KEEP>(one, src, c, qrow, lane);
        fma_group<ST>(one, a);
    }
#pragma unroll
    for (int g = 0; g < NQ; ++g) acc[g] = a[g];
}

// What happens to the 64 x NQ sums of an item: block maxima always, the scores themselves
// unless the running bound of the query says that nothing here can enter its top-k.
template <int ST, int NQ>
__device__ __forceinline__ void scan_finish(const ScanItem& it, int d, const float (&acc)[kQB],
                                            float* __restrict__ scores, float* __restrict__ bmax, int lane,
                                            unsigned long long* __restrict__ qthr, int prune_blocks,
                                            int prune_j) {
    constexpr int E = Store<ST>::E;
    const int nchunk = d / E;
    const int nq = (int)it.nq;
    const int ld_lane = min(lane, (int)it.nvalid - 1);
    float scale = 1.f;                              // int8: the lane's scale sits behind the codes
    if constexpr (ST == kI8)
        scale = *(reinterpret_cast<const float*>(static_cast<const char*>(it.data) + (size_t)nchunk * kLanes * 16) + ld_lane);
    const bool valid = lane < (int)it.nvalid;
#pragma unroll
    for (int g = 0; g < NQ; ++g) {
        if (g < nq) {
            const float s = valid ? (ST == kI8 ? acc[g] * scale : acc[g]) : -INFINITY;
            const uint32_t sb = it.sblk + (uint32_t)g * it.nblk;
            const float mx = wave_max(s, lane);
            bool store = true;
            if (prune_blocks) {
                // qthr[q] = (best, second best) over blocks of "j-th largest score in the
                // block"; with one block in play both halves are equal.  The low half is
                // a lower bound of q's k-th best score: >= k candidates reach it.
                unsigned long long* slot = qthr + it.q[g];
                const uint32_t thr = (uint32_t)__atomic_load_n(slot, __ATOMIC_RELAXED);
                const uint32_t omx = ord_of(mx);
                if (omx < thr) {
                    store = false;                 // nothing here can enter the top-k
                } else {
                    const uint32_t o = valid ? ord_of(s) : 0u;
                    uint32_t t = 0;                // j-th largest of the block, bit by bit; only its
                                                   // excess over the bound matters, and it exceeds
                                                   // the bound only if j scores of the block do
                    if (__popcll(__ballot(o > thr)) >= prune_j) {
                        for (int bit = 31; bit >= 0; --bit) {
                            const uint32_t cand = t | (1u << bit);
                            if (__popcll(__ballot(o >= cand)) >= prune_j) t = cand;
                        }
                    }
                    if (t > thr && lane == 0) {
                        if (prune_blocks == 1) {
                            atomicMax(slot, ((unsigned long long)t << 32) | t);
                        } else {
                            unsigned long long old = __atomic_load_n(slot, __ATOMIC_RELAXED);
                            for (;;) {
                                const uint32_t hi = (uint32_t)(old >> 32), lo = (uint32_t)old;
                                unsigned long long nw;
                                if (t > hi) nw = ((unsigned long long)t << 32) | hi;
                                else if (t > lo) nw = ((unsigned long long)hi << 32) | t;
                                else break;
                                const unsigned long long prev = atomicCAS(slot, old, nw);
                                if (prev == old) break;
                                old = prev;
                            }
                        }
                    }
                }
            }
            if (store) __builtin_nontemporal_store(s, scores + (size_t)sb * kLanes + lane);
            if (lane == 0) bmax[sb] = mx;
        }
    }
}

template <int ST, int U>
__device__ __forceinline__ void accumulate_dispatch(const ScanItem& it, const float* __restrict__ Q, int d,
                                                    int c0, int c1, int lane, float (&acc)[kQB]) {
    if (it.nq == 1) scan_accumulate<ST, 1, U>(it, Q, d, c0, c1, lane, acc);
    else if (it.nq == 2) scan_accumulate<ST, 2, U>(it, Q, d, c0, c1, lane, acc);
    else if (it.shared) scan_accumulate<ST, kQB, U, true>(it, Q, d, c0, c1, lane, acc);
    else scan_accumulate<ST, kQB, U>(it, Q, d, c0, c1, lane, acc);
}

template <int ST>
__device__ __forceinline__ void finish_dispatch(const ScanItem& it, int d, const float (&acc)[kQB],
                                                float* __restrict__ scores, float* __restrict__ bmax, int lane,
                                                unsigned long long* __restrict__ qthr, int prune_blocks,
                                                int prune_j) {
    if (it.nq == 1) scan_finish<ST, 1>(it, d, acc, scores, bmax, lane, qthr, prune_blocks, prune_j);
    else if (it.nq == 2) scan_finish<ST, 2>(it, d, acc, scores, bmax, lane, qthr, prune_blocks, prune_j);
    else scan_finish<ST, kQB>(it, d, acc, scores, bmax, lane, qthr, prune_blocks, prune_j);
}

template <int ST, int U>
__device__ __forceinline__ void scan_dispatch(const ScanItem& it, const float* __restrict__ Q,
                                              int d, float* __restrict__ scores,
                                              float* __restrict__ bmax, int lane,
                                              unsigned long long* __restrict__ qthr,
                                              int prune_blocks, int prune_j) {
    float acc[kQB];
    accumulate_dispatch<ST, U>(it, Q, d, 0, d / Store<ST>::E, lane, acc);
    finish_dispatch<ST>(it, d, acc, scores, bmax, lane, qthr, prune_blocks, prune_j);
}

// One item per group of SPLIT wavefronts of a 4-wavefront workgroup: wavefront p of the
// group takes the chunks [nchunk*p/SPLIT, nchunk*(p+1)/SPLIT) of the block, the partial sums
// meet in LDS and the first wavefront of the group adds them in ascending p and finishes the
// item.  Items become SPLIT times shorter and SPLIT times as many, which shortens the last,
// partly filled round of a plan with few items, and the wavefronts of a group read one
// contiguous region side by side.  The order of the additions differs from the unsplit
// kernel's, so an index uses one or the other throughout.
template <int ST, int U, int SPLIT>
__global__ __launch_bounds__(256) void k_scan_split(
    const ScanItem* __restrict__ items, const unsigned long long* __restrict__ n_items_dev,
    uint32_t n_items_host, const float* __restrict__ Q, int d, float* __restrict__ scores,
    float* __restrict__ bmax, unsigned long long* __restrict__ qthr, int prune_blocks, int prune_j) {
    static_assert(SPLIT == 2 || SPLIT == 4, "two or four wavefronts per item");
    __shared__ float part[4][kQB][kLanes];
    const int lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t T = n_items_dev ? (uint32_t)*n_items_dev : n_items_host;
    const uint32_t t = blockIdx.x * (4 / SPLIT) + wave / SPLIT;
    const uint32_t p = wave % SPLIT;
    const bool active = t < T;
    ScanItem it = items[active ? t : 0];
    float acc[kQB] = {0.f, 0.f, 0.f, 0.f};
    if (active) {
        const int nchunk = d / Store<ST>::E;
        accumulate_dispatch<ST, U>(it, Q, d, (int)(nchunk * p / SPLIT), (int)(nchunk * (p + 1) / SPLIT), lane, acc);
        if (p > 0) {
#pragma unroll
            for (int g = 0; g < kQB; ++g) part[wave][g][lane] = acc[g];
        }
    }
    __syncthreads();
    if (active && p == 0) {
#pragma unroll
        for (int o = 1; o < SPLIT; ++o)
#pragma unroll
            for (int g = 0; g < kQB; ++g) acc[g] += part[wave + o][g][lane];
        finish_dispatch<ST>(it, d, acc, scores, bmax, lane, qthr, prune_blocks, prune_j);
    }
}

constexpr int kScanWaves = 4;   // default wavefronts per workgroup of the scan

// One wavefront per item; the grid is sized by the host's upper bound on the items and the
// wavefronts beyond the real count leave at once.  The item count comes from device memory
// (n_items_dev) when the plan was made on the device, else from the host (n_items_host).
template <int ST, int U, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void k_scan(
    const ScanItem* __restrict__ items, const unsigned long long* __restrict__ n_items_dev,
    uint32_t n_items_host, const float* __restrict__ Q, int d, float* __restrict__ scores,
    float* __restrict__ bmax, unsigned long long* __restrict__ qthr, int prune_blocks, int prune_j) {
    const int lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t T = n_items_dev ? (uint32_t)*n_items_dev : n_items_host;
    const uint32_t t = blockIdx.x * WAVES + wave;
    if (t >= T) return;
    ScanItem it = items[t];
    scan_dispatch<ST, U>(it, Q, d, scores, bmax, lane, qthr, prune_blocks, prune_j);
}

// Upload-time re-layout: row-major rows of a piece of the index -> blocked storage.
// A row is `row_bytes - tail_bytes` bytes of elements (a multiple of 16) followed by
// `tail_bytes` (0, or 4: the scale of an int8 record); a block holds the element chunks
// of its 64 vectors and then their 64 tails.  grid.x = list within the piece, grid.y =
// block within the list.
__global__ __launch_bounds__(256) void k_relayout(const char* __restrict__ src_rows,
                                                  const int64_t* __restrict__ offsets,
                                                  const void* const* __restrict__ list_ptr,
                                                  int64_t list_begin, int row_bytes, int tail_bytes) {
    const int64_t l = list_begin + blockIdx.x;
    const int64_t len = offsets[l + 1] - offsets[l];
    const int64_t b = blockIdx.y;
    if (b * kLanes >= len) return;
    const int64_t row0 = offsets[l] - offsets[list_begin] + b * kLanes;
    const int nchunk = (row_bytes - tail_bytes) / 16;
    char* blk = static_cast<char*>(const_cast<void*>(list_ptr[l])) + (size_t)b * kLanes * (size_t)row_bytes;
    if (tail_bytes == 0) {                   // rows are 16-byte aligned
        u4* dst = reinterpret_cast<u4*>(blk);
        for (int u = threadIdx.x; u < nchunk * kLanes; u += 256) {
            int c = u / kLanes, lane = u % kLanes;
            u4 v = {0u, 0u, 0u, 0u};
            if (b * kLanes + lane < len)
                v = *reinterpret_cast<const u4*>(src_rows + (size_t)(row0 + lane) * row_bytes + (size_t)c * 16);
            dst[u] = v;
        }
    } else {                                 // rows are 4-byte aligned: word by word
        unsigned* dst = reinterpret_cast<unsigned*>(blk);
        for (int u = threadIdx.x; u < nchunk * kLanes * 4; u += 256) {
            int c = u / (kLanes * 4), lane = (u / 4) % kLanes, wd = u % 4;
            unsigned v = 0u;
            if (b * kLanes + lane < len)
                v = *reinterpret_cast<const unsigned*>(src_rows + (size_t)(row0 + lane) * row_bytes + (size_t)c * 16 + wd * 4);
            dst[u] = v;
        }
        unsigned* tails = dst + (size_t)nchunk * kLanes * 4;
        const int tw = tail_bytes / 4;
        for (int u = threadIdx.x; u < kLanes * tw; u += 256) {
            int lane = u / tw, wd = u % tw;
            unsigned v = 0u;
            if (b * kLanes + lane < len)
                v = *reinterpret_cast<const unsigned*>(src_rows + (size_t)(row0 + lane) * row_bytes + (row_bytes - tail_bytes) + wd * 4);
            tails[u] = v;
        }
    }
}

// Inverse of k_relayout for one list (debug read-back).
__global__ __launch_bounds__(256) void k_unlayout(const char* __restrict__ blocks, int64_t len,
                                                  int row_bytes, int tail_bytes, char* __restrict__ dst_rows) {
    const int64_t b = blockIdx.x;
    const int nchunk = (row_bytes - tail_bytes) / 16;
    const unsigned* src = reinterpret_cast<const unsigned*>(blocks + (size_t)b * kLanes * (size_t)row_bytes);
    for (int u = threadIdx.x; u < nchunk * kLanes * 4; u += 256) {
        int c = u / (kLanes * 4), lane = (u / 4) % kLanes, wd = u % 4;
        if (b * kLanes + lane < len)
            *reinterpret_cast<unsigned*>(dst_rows + (size_t)(b * kLanes + lane) * row_bytes + (size_t)c * 16 + wd * 4) = src[u];
    }
    const unsigned* tails = src + (size_t)nchunk * kLanes * 4;
    const int tw = tail_bytes / 4;
    for (int u = threadIdx.x; u < kLanes * tw; u += 256) {
        int lane = u / tw, wd = u % tw;
        if (b * kLanes + lane < len)
            *reinterpret_cast<unsigned*>(dst_rows + (size_t)(b * kLanes + lane) * row_bytes + (row_bytes - tail_bytes) + wd * 4) = tails[u];
    }
}

// Plain streaming copy, 16 bytes per lane and step (counter calibration).
__global__ __launch_bounds__(256) void k_copy_u4(u4* __restrict__ dst, const u4* __restrict__ src, size_t n) {
    size_t i = blockIdx.x * (size_t)256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i < n; i += stride) dst[i] = src[i];
}

// Plain streaming read with the scan's access pattern and nothing else: one wavefront
// per contiguous 96 KiB tile, two buffers of 8 nontemporal 16-byte loads per lane.  Its
// rate is the practical ceiling for the scan on this machine.  `sink` is never written
// unless the data XORs to a magic value (keeps the loads alive).
__global__ __launch_bounds__(256) void k_read_tiles(const u4* __restrict__ base, size_t ntiles,
                                                    unsigned* __restrict__ sink) {
    constexpr int U = 8, kTileU4 = 6144, kSteps = kTileU4 / kLanes;   // 96 loads per lane
    size_t t = blockIdx.x * (size_t)4 + (threadIdx.x >> 6);
    if (t >= ntiles) return;
    const int lane = threadIdx.x & 63;
    gptr_u4 src = (gptr_u4)(uintptr_t)(base + t * kTileU4) + lane;
    u4 acc = {0u, 0u, 0u, 0u};
    u4 a[U], b[U];
#pragma unroll
    for (int u = 0; u < U; ++u) a[u] = __builtin_nontemporal_load(src + u * kLanes);
    for (int g = 0; g + 2 <= kSteps / U; g += 2) {
#pragma unroll
        for (int u = 0; u < U; ++u) b[u] = __builtin_nontemporal_load(src + ((g + 1) * U + u) * kLanes);
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= a[u];
        if (g + 2 < kSteps / U) {
#pragma unroll
            for (int u = 0; u < U; ++u) a[u] = __builtin_nontemporal_load(src + ((g + 2) * U + u) * kLanes);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= b[u];
    }
    unsigned r = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (r == 0x9e3779b9u) sink[0] = r;
}

__global__ void k_iota_u32(uint32_t* __restrict__ p, size_t n) {
    size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
    if (i < n) p[i] = (uint32_t)i;
}

// rank_of_pos[pos_sorted[r]] = r
__global__ void k_scatter_rank(const uint32_t* __restrict__ pos_sorted, uint32_t* __restrict__ rank_of_pos,
                               size_t n) {
    size_t r = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
    if (r < n) rank_of_pos[pos_sorted[r]] = (uint32_t)r;
}

// ids[pos] = id_sorted[rank_of_pos[pos]] for pos in [pos_begin, pos_begin+count)
__global__ void k_gather_ids(const int64_t* __restrict__ id_sorted, const uint32_t* __restrict__ rank_of_pos,
                             int64_t pos_begin, int64_t count, int64_t* __restrict__ out) {
    int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (i < count) out[i] = id_sorted[rank_of_pos[pos_begin + i]];
}

}  // namespace ivf
