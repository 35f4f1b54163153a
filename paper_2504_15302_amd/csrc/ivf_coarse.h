// Coarse quantisation: S = Q * C^T in fp32 on the matrix cores, plus the maximum of
// every tile of 32 centroid scores (the first level of the probe selection).
//
// One wavefront owns 32 centroids and up to MT*32 queries and runs the whole K loop
// with v_mfma_f32_32x32x2_f32.  The centroid operand is private to the wavefront and
// is loaded straight from HBM (each centroid row is read exactly once per query
// chunk); the query operand is shared by the four wavefronts of the workgroup and is
// staged through LDS.  Both operands are K-contiguous in memory, so a lane loads four
// consecutive k at once and feeds them to four consecutive MFMA steps; the two lane
// halves take the two k of a step from columns 4 apart.  The sum over k does not
// depend on that assignment as long as both operands use the same one.
#pragma once
#include "ivf_device.h"

namespace ivf {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kCoarseKT = 32;    // k per pipeline step
constexpr int kCoarseLd = 36;    // LDS row stride in floats (32 + 4: keeps b128 reads conflict-free)
constexpr int kCoarseNT = 128;   // centroids per workgroup (4 wavefronts x 32)

template <int MT>
__global__ __launch_bounds__(256) void k_coarse(const float* __restrict__ Q,
                                                const float* __restrict__ C,
                                                float* __restrict__ S, float* __restrict__ tmax,
                                                int nq, int nlist, int d, int ntile) {
    __shared__ float qs[MT * 32 * kCoarseLd];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int col = lane & 31;
    const int half = lane >> 5;
    const int m0 = blockIdx.y * (MT * 32);
    const int n0 = blockIdx.x * kCoarseNT + wave * 32;
    const int n = n0 + col;
    const bool n_ok = n < nlist;
    const float* crow = C + (size_t)(n_ok ? n : nlist - 1) * d;

    v16f acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mt][v] = 0.f;

    // Software pipeline over k: the centroid operand and the query tile of step i+1 are
    // loaded into registers while the MFMAs of step i run, so the HBM/L2 latency hides
    // behind 16*MT matrix instructions per wavefront.
    // All loads are unconditional (addresses clamped into range, so the loads of a
    // step issue back to back); rows past nq / nlist produce values that are never
    // stored, and a k past d (d not a multiple of 32) is zeroed in the centroid operand.
    auto load_b = [&](v4f (&b)[4], int kb) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int kk = kb + j * 8 + half * 4;
            b[j] = *reinterpret_cast<const v4f*>(crow + min(kk, d - 4));
        }
    };
    auto mask_b = [&](v4f (&b)[4], int kb) {        // applied when the values are first used
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (kb + j * 8 + half * 4 >= d) b[j] = v4f{0.f, 0.f, 0.f, 0.f};
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
    auto read_a = [&](v4f (&a)[MT], int j) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            a[mt] = *reinterpret_cast<const v4f*>(&qs[(mt * 32 + col) * kCoarseLd + j * 8 + half * 4]);
    };
    v4f b_cur[4], b_nxt[4], q_reg[MT];
    load_b(b_cur, 0);
    mask_b(b_cur, 0);
    load_q(q_reg, 0);
    for (int kb = 0; kb < d; kb += kCoarseKT) {
        __syncthreads();                    // the previous step's LDS reads are done
#pragma unroll
        for (int i = 0; i < MT; ++i) {
            int idx = threadIdx.x + i * 256;
            int row = idx >> 3, c4 = idx & 7;
            *reinterpret_cast<v4f*>(&qs[row * kCoarseLd + c4 * 4]) = q_reg[i];
        }
        __syncthreads();
        const int kn = min(kb + kCoarseKT, d - 4);   // last step: a harmless reload
        load_b(b_nxt, kn);
        load_q(q_reg, kn);
        __builtin_amdgcn_sched_barrier(0);   // keep these loads ahead of the MFMAs that hide them
        v4f a_cur[MT], a_nxt[MT];
        read_a(a_cur, 0);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (j < 3) read_a(a_nxt, j + 1);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    acc[mt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_cur[mt][s], b_cur[j][s], acc[mt], 0, 0, 0);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) a_cur[mt] = a_nxt[mt];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) b_cur[j] = b_nxt[j];
        mask_b(b_cur, kb + kCoarseKT);
    }

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
