// Scan of inverted lists stored as product-quantisation codes (the memory-for-accuracy
// trade that the paper's on-disk index variant makes, Section 6.5 "On-Disk Index").
// A stored vector is M one-byte codes; code m selects one of 256 codewords of subspace m
// (d/M consecutive dimensions) and the vector stands for the concatenation of its
// codewords.  The inner product with a query is then a sum of M table entries:
//   T[q][m][c] = <q_m, B[m][c]>          (k_pq_tables, once per search)
//   score(q, i) = sum_m T[q][m][code_im] (k_pq_scan, ascending m, fp32)
// Codes use the blocked layout of the other storage types ([16-code chunks][64 lanes][16
// bytes], a lane owns a vector); one workgroup handles one (query, list) pair with the
// query's table in LDS (M KiB) and writes block maxima and scores exactly like the flat
// scan, so the final selection is shared.  The kernel is bound by the LDS gathers (64
// random 4-byte reads per code byte and wavefront), not by HBM: the codes are a sixteenth
// of the fp16 bytes.
#pragma once
#include "ivf_scan.h"

namespace ivf {

constexpr int kPqThreads = 512;     // workgroup of the code scan: eight wavefronts share one table
constexpr int kPqMaxM = 128;        // subspaces: the table of one query must fit LDS (1 KiB each)

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

// One workgroup per (query, list) pair, numbered like the regrouping numbers them (by
// list, then query).  Dynamic LDS: M * 256 floats.
__global__ __launch_bounds__(kPqThreads) void k_pq_scan(
    const uint32_t* __restrict__ pair_flat, const int32_t* __restrict__ probes,
    const uint32_t* __restrict__ pair_start, const uint32_t* __restrict__ sblk_start,
    const int32_t* __restrict__ nblk, const int32_t* __restrict__ len,
    const void* const* __restrict__ list_ptr, int nprobe, int M,
    const float* __restrict__ tables, float* __restrict__ scores, float* __restrict__ bmax,
    unsigned long long* __restrict__ qthr, int prune_blocks, int prune_j) {
    extern __shared__ float lut[];                        // [M][256] of this pair's query
    const uint32_t pi = blockIdx.x;
    const uint32_t f = pair_flat[pi];                     // slot of the pair in the probe table
    const int q = (int)(f / (uint32_t)nprobe);
    const int l = probes[f];
    const char* base = reinterpret_cast<const char*>(reinterpret_cast<uintptr_t>(list_ptr[l]) & ~(uintptr_t)1);
    const int nb = nblk[l];
    if (!base || nb == 0) return;                         // the whole workgroup leaves together
    const uint32_t sb0 = sblk_start[l] + (pi - pair_start[l]) * (uint32_t)nb;
    {
        const f4* src = reinterpret_cast<const f4*>(tables + (size_t)q * M * 256);
        f4* dst = reinterpret_cast<f4*>(lut);
        for (int i = threadIdx.x; i < M * 64; i += kPqThreads) dst[i] = src[i];
    }
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int ln = len[l];
    const int nchunk = M / 16;
    for (int b = wave; b < nb; b += kPqThreads / 64) {
        ScanItem it;
        it.data = nullptr;
        it.sblk = sb0 + (uint32_t)b;
        it.nblk = (uint32_t)nb;
        it.q[0] = it.q[1] = it.q[2] = it.q[3] = (uint16_t)q;
        it.nq = 1;
        it.nvalid = (uint16_t)min(64, ln - b * 64);
        it.pad = 0;
        // lanes past the end of the list re-read the last valid vector; discarded in scan_finish
        const int ld_lane = min(lane, (int)it.nvalid - 1);
        const gptr_u4 blk = (gptr_u4)(uintptr_t)(base + (size_t)b * kLanes * M) + ld_lane;
        float acc[kQB] = {0.f, 0.f, 0.f, 0.f};
        for (int ch = 0; ch < nchunk; ++ch) {
            const u4 v = __builtin_nontemporal_load(blk + (size_t)ch * kLanes);
            const float* t = lut + (size_t)ch * 16 * 256;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const unsigned code = (v[j / 4] >> (8 * (j % 4))) & 255u;
                acc[0] += t[j * 256 + code];
            }
        }
        scan_finish<kF32, 1>(it, 0, acc, scores, bmax, lane, qthr, prune_blocks, prune_j);
    }
}

}  // namespace ivf
