// Scan of inverted lists stored as product-quantisation codes (the memory-for-accuracy
// trade that the paper's on-disk index variant makes, Section 6.5 "On-Disk Index").
// A stored vector is M one-byte codes; code m selects one of 256 codewords of subspace m
// (d/M consecutive dimensions) and the vector stands for the concatenation of its
// codewords.  The inner product with a query is then a sum of M table entries:
//   T[q][m][c] = <q_m, B[m][c]>          (k_pq_tables, once per search)
//   score(q, i) = sum_m T[q][m][code_im] (k_pq_scan, ascending m, fp32)
// Codes use the blocked layout of the other storage types ([16-code chunks][64 lanes][16
// bytes], a lane owns a vector).  A workgroup of sixteen wavefronts holds one query's table
// in LDS (M KiB) and scans a share of that query's probed lists, block after block, each
// wavefront fetching its next block while it gathers for the current one; it writes block
// maxima and scores exactly like the flat scan, so the final selection is shared.  The
// kernel is bound by the LDS gathers (64 random 4-byte reads per code byte and wavefront),
// not by HBM: the codes are a sixteenth of the fp16 bytes.
#pragma once
#include "ivf_scan.h"

namespace ivf {

constexpr int kPqThreads = 1024;    // workgroup of the code scan: sixteen wavefronts share one table
constexpr int kPqMaxM = 128;        // subspaces: the table of one query must fit LDS (1 KiB each)
constexpr int kPqWgLists = 16;      // most lists that one workgroup takes
constexpr int kPqMaxChunks = kPqMaxM / 16;

// grid (M, nq), 256 threads: thread c computes T[q][m][c] over the d/M dimensions of
// subspace m in ascending order.
__global__ __launch_bounds__(256) void k_pq_tables(const float* __restrict__ Q,
                                                   const float* __restrict__ codebooks,
                                                   float* __restrict__ tables, int d, int M) {
    const int m = blockIdx.x, q = blockIdx.y, c = threadIdx.x;
    const int dsub = d / M;
    const float* qm = Q + (size_t)q * d + (size_t)m * dsub;
    const float* b = codebooks + ((size_t)m * 256 + c) * dsub;
    float s = 0.f;
    for (int t = 0; t < dsub; ++t) s = __builtin_fmaf(qm[t], b[t], s);
    tables[((size_t)q * M + m) * 256 + c] = s;
}

// The 16-byte chunks of one block of codes, one vector per lane (lanes past the end of
// the list re-read the last valid vector; their sums are discarded by scan_finish).
__device__ __forceinline__ void pq_load_block(u4 (&buf)[kPqMaxChunks], const char* base, int b, int ln, int M,
                                              int nchunk, int lane) {
    const int nvalid = min(64, ln - b * 64);
    const gptr_u4 blk = (gptr_u4)(uintptr_t)(base + (size_t)b * kLanes * M) + min(lane, nvalid - 1);
#pragma unroll
    for (int ch = 0; ch < kPqMaxChunks; ++ch)
        if (ch < nchunk) buf[ch] = __builtin_nontemporal_load(blk + (size_t)ch * kLanes);
}

// grid (parts, nq): workgroup (p, q) takes the probes [nprobe*p/parts, nprobe*(p+1)/parts)
// of query q (at most kPqWgLists of them) and treats their blocks as one sequence, which
// its wavefronts take in turn.  Dynamic LDS: M * 256 floats.
__global__ __launch_bounds__(kPqThreads) void k_pq_scan(
    const int32_t* __restrict__ probes, const uint32_t* __restrict__ pair_of_probe,
    const uint32_t* __restrict__ pair_start, const uint32_t* __restrict__ sblk_start,
    const int32_t* __restrict__ nblk, const int32_t* __restrict__ len,
    const void* const* __restrict__ list_ptr, int nprobe, int M,
    const float* __restrict__ tables, float* __restrict__ scores, float* __restrict__ bmax,
    unsigned long long* __restrict__ qthr, int prune_blocks, int prune_j) {
    extern __shared__ float lut[];                        // [M][256] of this workgroup's query
    __shared__ const char* l_base[kPqWgLists];
    __shared__ int l_nb[kPqWgLists], l_len[kPqWgLists];
    __shared__ uint32_t l_sb0[kPqWgLists];
    const int q = blockIdx.y;
    const int j0 = (int)((long long)nprobe * blockIdx.x / gridDim.x);
    const int nl = (int)((long long)nprobe * (blockIdx.x + 1) / gridDim.x) - j0;
    if ((int)threadIdx.x < nl) {
        const size_t f = (size_t)q * nprobe + j0 + threadIdx.x;   // slot in the probe table
        const int l = probes[f];
        const char* base = reinterpret_cast<const char*>(reinterpret_cast<uintptr_t>(list_ptr[l]) & ~(uintptr_t)1);
        const int nb = base ? nblk[l] : 0;
        l_base[threadIdx.x] = base;
        l_nb[threadIdx.x] = nb;
        l_len[threadIdx.x] = len[l];
        l_sb0[threadIdx.x] = sblk_start[l] + (pair_of_probe[f] - pair_start[l]) * (uint32_t)nb;
    }
    {
        const f4* src = reinterpret_cast<const f4*>(tables + (size_t)q * M * 256);
        f4* dst = reinterpret_cast<f4*>(lut);
        for (int i = threadIdx.x; i < M * 64; i += kPqThreads) dst[i] = src[i];
    }
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    constexpr int kWaves = kPqThreads / 64;
    const int nchunk = M / 16;
    int total = 0;
    for (int i = 0; i < nl; ++i) total += l_nb[i];
    // (li, first): the list that holds block g of the sequence and the number of its first block
    int li = 0, first = 0;
    auto seek = [&](int g) {
        while (li < nl && g >= first + l_nb[li]) { first += l_nb[li]; ++li; }
    };
    u4 cur[kPqMaxChunks], nxt[kPqMaxChunks];
    int g = wave;
    if (g < total) {
        seek(g);
        pq_load_block(cur, l_base[li], g - first, l_len[li], M, nchunk, lane);
    }
    while (g < total) {
        const int ci = li, cb = g - first;                // the block in `cur`
        const int gn = g + kWaves;
        if (gn < total) {
            seek(gn);
            pq_load_block(nxt, l_base[li], gn - first, l_len[li], M, nchunk, lane);
        }
        float acc[kQB] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ch = 0; ch < kPqMaxChunks; ++ch) {
            if (ch < nchunk) {
                const float* t = lut + (size_t)ch * 16 * 256;
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const unsigned code = (cur[ch][j / 4] >> (8 * (j % 4))) & 255u;
                    acc[0] += t[j * 256 + code];
                }
            }
        }
        ScanItem it;
        it.data = nullptr;
        it.sblk = l_sb0[ci] + (uint32_t)cb;
        it.nblk = (uint32_t)l_nb[ci];
        it.q[0] = it.q[1] = it.q[2] = it.q[3] = (uint16_t)q;
        it.nq = 1;
        it.nvalid = (uint16_t)min(64, l_len[ci] - cb * 64);
        it.shared = 0;
        scan_finish<kF32, 1>(it, 0, acc, scores, bmax, lane, qthr, prune_blocks, prune_j);
        if (gn < total) {
#pragma unroll
            for (int ch = 0; ch < kPqMaxChunks; ++ch)
                if (ch < nchunk) cur[ch] = nxt[ch];
        }
        g = gn;
    }
}

}  // namespace ivf
