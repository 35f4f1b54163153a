// Coarse quantisation: S = Q * C^T in fp32 on the matrix cores, plus the maximum of
// every tile of 32 centroid scores (the first level of the probe selection).
//
// One wavefront owns 32 centroids and up to MT*32 queries and runs the whole K loop
// with v_mfma_f32_32x32x2_f32.  The centroid operand is private to the wavefront and
// is loaded straight from HBM (each centroid row is read exactly once per query
// chunk); the query operand is shared by the four wavefronts of the workgroup and is
// staged through LDS.  A lane holds four consecutive k of its row and feeds them to four
// consecutive MFMA steps; the two lane halves take the two k of a step from columns 4
// apart.  The sum over k does not depend on that assignment as long as both operands
// use the same one.
//
// The library keeps the centroids in the order this kernel reads them: for every tile of
// 32 centroids and every step of 32 k, one contiguous 4 KiB piece laid out as
// [j = 0..3][lane half][centroid in tile][4 floats], so that each of the wavefront's four
// load instructions of a step fetches 1 KiB of consecutive bytes (row-major centroids
// gave 32 scattered 32-byte pieces per instruction and kept the matrix cores waiting
// for HBM).  Rows past nlist and k past d are stored as zeros.
#pragma once
#include "ivf_device.h"

namespace ivf {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kCoarseKT = 32;    // k per pipeline step
constexpr int kCoarseLd = 36;    // LDS row stride in floats (32 + 4: keeps b128 reads conflict-free)
constexpr int kCoarseNT = 128;   // centroids per workgroup (4 wavefronts x 32)

// Row-major centroids [nlist, d] -> the tiled order described above; one thread per 16 bytes.
__global__ void k_tile_centroids(const float* __restrict__ C, float* __restrict__ Ct, int nlist, int d,
                                 int nstep, size_t n_vec4) {
    const size_t o = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
    if (o >= n_vec4) return;
    const int col = (int)(o & 31), half = (int)((o >> 5) & 1), j = (int)((o >> 6) & 3);
    const size_t ts = o >> 8;                           // tile * nstep + step
    const int step = (int)(ts % (size_t)nstep);
    const size_t tile = ts / (size_t)nstep;
    const size_t row = tile * 32 + col;
    const int k = step * kCoarseKT + j * 8 + half * 4;
    v4f v = {0.f, 0.f, 0.f, 0.f};
    if (row < (size_t)nlist && k < d) v = *reinterpret_cast<const v4f*>(C + row * (size_t)d + k);
    reinterpret_cast<v4f*>(Ct)[o] = v;
}

template <int MT>
__global__ __launch_bounds__(256) void k_coarse(const float* __restrict__ Q,
                                                const float* __restrict__ Ct,
                                                float* __restrict__ S, float* __restrict__ tmax,
                                                int nq, int nlist, int d, int ntile,
                                                int* __restrict__ zero, int nzero) {
    // The search's zero-initialised scratch (probe histogram, cursors, counters, bounds) is
    // first touched by the kernels after this one: clearing it here saves a launch.
    for (size_t i = ((size_t)blockIdx.y * gridDim.x + blockIdx.x) * 256 + threadIdx.x; i < (size_t)nzero;
         i += (size_t)gridDim.x * gridDim.y * 256)
        zero[i] = 0;
    __shared__ float qs[2][MT * 32 * kCoarseLd];     // query tiles of two consecutive steps
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int col = lane & 31;
    const int half = lane >> 5;
    const int m0 = blockIdx.y * (MT * 32);
    const int n0 = blockIdx.x * kCoarseNT + wave * 32;
    const int n = n0 + col;
    const bool n_ok = n < nlist;
    const int nstep = (d + kCoarseKT - 1) / kCoarseKT;
    // a wavefront past the last tile (nlist not a multiple of 128) re-reads the last one; nothing of it is stored
    const v4f* ctile = reinterpret_cast<const v4f*>(Ct) + (size_t)min(n0 / 32, ntile - 1) * nstep * 256 + half * 32 + col;

    v16f acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mt][v] = 0.f;

    // Software pipeline over k: the centroid operand and the query tile of later steps are
    // loaded into registers while the MFMAs of step i run (16*MT matrix instructions per
    // wavefront and step).
    // All loads are unconditional (addresses clamped into range, so the loads of a step
    // issue back to back); rows past nq produce values that are never stored, and a k past
    // d (d not a multiple of 32) meets a stored zero in the centroid operand.
    auto load_b = [&](v4f (&b)[4], int step) {
        const v4f* p = ctile + (size_t)min(step, nstep - 1) * 256;
#pragma unroll
        for (int j = 0; j < 4; ++j) b[j] = p[j * 64];
    };
    auto load_q = [&](v4f (&qr)[MT], int kb) {
#pragma unroll
        for (int i = 0; i < MT; ++i) {
            int idx = threadIdx.x + i * 256;
            int row = idx >> 3, c4 = idx & 7;
            int m = min(m0 + row, nq - 1), kk = min(kb + c4 * 4, d - 4);
            qr[i] = *reinterpret_cast<const v4f*>(Q + (size_t)m * d + kk);
        }
    };
    auto read_a = [&](v4f (&a)[MT], const float* tile, int j) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            a[mt] = *reinterpret_cast<const v4f*>(&tile[(mt * 32 + col) * kCoarseLd + j * 8 + half * 4]);
    };
    // The centroid operand streams from HBM (every row is read once), whose latency under
    // load exceeds one step of MFMAs: it is fetched two steps ahead, into three register
    // sets that swap roles (the loop is unrolled by three, so no set is ever copied while
    // its loads are in flight).  The query tile comes from L2 and is fetched one step ahead.
    // Loads complete in issue order as far as the wait counter can tell: the query tile,
    // needed first, is issued first, so that waiting for it at the top of the next step
    // does not also wait for the centroid loads issued in the same step.
    v4f q_reg[MT];
    auto step = [&](v4f (&b_cur)[4], v4f (&b_far)[4], int kb) {
        // Two LDS tiles alternate, so one barrier per step is enough: a wavefront that has
        // passed the barrier of step s has seen every wavefront finish reading the tile of
        // step s-1, which is the one step s+1 overwrites.
        float* tile = qs[(kb / kCoarseKT) & 1];
#pragma unroll
        for (int i = 0; i < MT; ++i) {
            int idx = threadIdx.x + i * 256;
            int row = idx >> 3, c4 = idx & 7;
            *reinterpret_cast<v4f*>(&tile[row * kCoarseLd + c4 * 4]) = q_reg[i];
        }
        __syncthreads();
        load_q(q_reg, min(kb + kCoarseKT, d - 4));
        load_b(b_far, kb / kCoarseKT + 2);                 // past the end: a harmless reload
        __builtin_amdgcn_sched_barrier(0);   // keep these loads ahead of the MFMAs that hide them
        // LDS reads of the next eight k are issued before the MFMAs of the current eight, in
        // two alternating register sets; the group barriers below pin that order (left
        // alone, the scheduler gathers the reads and then waits for them in front of the
        // matrix instructions).
        v4f a[2][MT];
        read_a(a[0], tile, 0);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (j < 3) read_a(a[(j + 1) & 1], tile, j + 1);
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    acc[mt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[j & 1][mt][s], b_cur[j][s], acc[mt], 0, 0, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x100, 2 * MT, 0);     // reads for k 0..15
        __builtin_amdgcn_sched_group_barrier(0x008, 4 * MT, 0);     // MFMAs of k 0..7
        __builtin_amdgcn_sched_group_barrier(0x100, MT, 0);         // reads for k 16..23
        __builtin_amdgcn_sched_group_barrier(0x008, 4 * MT, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, MT, 0);         // reads for k 24..31
        __builtin_amdgcn_sched_group_barrier(0x008, 8 * MT, 0);
    };
    v4f b0[4], b1[4], b2[4];
    load_q(q_reg, 0);
    load_b(b0, 0);
    load_b(b1, 1);
    int st = 0;
    for (; st + 3 <= nstep; st += 3) {
        step(b0, b2, st * kCoarseKT);
        step(b1, b0, (st + 1) * kCoarseKT);
        step(b2, b1, (st + 2) * kCoarseKT);
    }
    if (st < nstep) step(b0, b2, st * kCoarseKT);                   // one or two steps are left
    if (st + 1 < nstep) step(b1, b0, (st + 1) * kCoarseKT);

    // accumulator element v of a lane is row 8*(v/4) + 4*half + v%4, column `col`
    const int tile = n0 / kCoarseTile;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            int m = m0 + mt * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
            float s = n_ok ? acc[mt][v] : -INFINITY;
            if (m < nq && n_ok) S[(size_t)m * nlist + n] = s;
            float mx = s;
#pragma unroll
            for (int o = 16; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
            if (col == 0 && m < nq && tile < ntile) tmax[(size_t)m * ntile + tile] = mx;
        }
    }
}

}  // namespace ivf
