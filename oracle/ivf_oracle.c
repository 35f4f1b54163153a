/*
 * CPU ORACLE for batched IVF inner-product top-k retrieval.  TEST INFRASTRUCTURE ONLY:
 * it is called by the tests, by the smoke check and by the benchmark's cpu_baseline
 * leg, never by the product path, and shares no code with the HIP library.
 *
 * What it computes is the plain definition of the retrieval step of a
 * retrieve-then-generate pipeline: the stored chunk embeddings are matched with the
 * query embedding by similarity search (paper Section 2.2, "On-demand RAG Serving"),
 * a batch of query vectors per call (Section 2.3, "Batch Scheduling"), the top-k most
 * relevant chunks are returned (Section 6.1, "Workloads"), and no approximation or
 * truncation is allowed to change the outcome (Section 6.1, "Key Metrics").  The paper
 * leaves index type and metric open; the benchmark fixes them: IVF-Flat, inner
 * product, given centroids.
 *
 *   coarse      c(q,j) = sum_t Q[q,t]*C[j,t]                       fp64, t ascending
 *   probes      the nprobe lists with largest c(q,.), ties -> smaller list number
 *   scan        s(q,i) = sum_t Q[q,t]*X[i,t] for every i in a probed list, fp64,
 *               t ascending; fp16 storage is widened exactly before multiplying;
 *               int8 storage (a record of d signed codes and one fp32 scale per
 *               vector, standing for the vector scale*codes) gives
 *               s(q,i) = scale_i * sum_t Q[q,t]*code[i,t]
 *   select      candidates ordered by (s descending, user id ascending, position
 *               ascending); the first kout are reported, the rest padded (-1, -inf)
 *   assign      list of a vector = arg-max_j <x, C_j>, ties -> smaller j
 *
 * Nothing is blocked, fused or reordered.  OpenMP only distributes independent
 * (query) or (vector) iterations over threads; each sum is still one sequential loop.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* IEEE binary16 -> double, exact.  sign(1) exponent(5, bias 15) fraction(10). */
double oracle_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);              /* subnormal: f * 2^-10 * 2^-14 */
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)f / 1024.0, e - 15);
    return sign ? -v : v;
}

int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static inline double elem(const void *x, int dtype, int64_t idx)
{
    if (dtype == 0)
        return (double)((const float *)x)[idx];
    return oracle_half_to_double(((const uint16_t *)x)[idx]);
}

/* <q, stored vector i> in fp64, t ascending.  dtype 2: rows are records of d int8 codes
   followed by the vector's fp32 scale (d+4 bytes); the stored vector is scale*codes. */
static double stored_dot(const void *X, int dtype, int64_t i, int d, const float *q)
{
    double s = 0.0;
    if (dtype == 2) {
        const unsigned char *row = (const unsigned char *)X + (size_t)i * ((size_t)d + 4);
        float scale;
        for (int t = 0; t < d; ++t)
            s += (double)q[t] * (double)(signed char)row[t];
        memcpy(&scale, row + d, sizeof scale);
        return (double)scale * s;
    }
    for (int t = 0; t < d; ++t)
        s += (double)q[t] * elem(X, dtype, i * d + t);
    return s;
}

/* coarse[q*nlist + j] = <Q_q, C_j> in fp64 */
int oracle_coarse(const float *Q, int64_t nq, const float *C, int64_t nlist, int d, double *coarse)
{
    if (!Q || !C || !coarse || nq < 0 || nlist < 0 || d <= 0)
        return -1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t q = 0; q < nq; ++q)
        for (int64_t j = 0; j < nlist; ++j) {
            double s = 0.0;
            for (int t = 0; t < d; ++t)
                s += (double)Q[q * d + t] * (double)C[j * d + t];
            coarse[q * nlist + j] = s;
        }
    return 0;
}

typedef struct {
    double s;
    int64_t id;
    int64_t pos;
} cand_t;

/* best first: larger score, then smaller id, then smaller position */
static int cand_cmp(const void *a, const void *b)
{
    const cand_t *x = (const cand_t *)a, *y = (const cand_t *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    if (x->id < y->id) return -1;
    if (x->id > y->id) return 1;
    if (x->pos < y->pos) return -1;
    if (x->pos > y->pos) return 1;
    return 0;
}

/* probes[q*nprobe + r] = list with the (r+1)-th largest coarse score, ties -> smaller j.
 * nprobe must be <= nlist. */
int oracle_probe_select(const double *coarse, int64_t nq, int64_t nlist, int nprobe, int32_t *probes)
{
    if (!coarse || !probes || nprobe <= 0 || nprobe > nlist)
        return -1;
    int err = 0;
#pragma omp parallel for schedule(dynamic)
    for (int64_t q = 0; q < nq; ++q) {
        cand_t *c = (cand_t *)malloc(sizeof(cand_t) * (size_t)nlist);
        if (!c) { err = 1; continue; }
        for (int64_t j = 0; j < nlist; ++j) {
            c[j].s = coarse[q * nlist + j];
            c[j].id = j;
            c[j].pos = j;
        }
        qsort(c, (size_t)nlist, sizeof(cand_t), cand_cmp);
        for (int r = 0; r < nprobe; ++r)
            probes[q * nprobe + r] = (int32_t)c[r].id;
        free(c);
    }
    return err ? -2 : 0;
}

/* Exact scan of the given probe lists and sorted selection of the kout best.
 *   X        [n, d] list-major rows, dtype 0 = float32, 1 = IEEE binary16,
 *            2 = [n] records of d int8 codes + fp32 scale
 *   ids      [n] user ids; offsets [nlist+1]
 *   probes   [nq, nprobe] list numbers (a negative entry is skipped)
 *   out_ids  [nq, kout], out_scores [nq, kout] fp64 (pad: -1, -inf)
 */
int oracle_scan_select(const void *X, int dtype, const int64_t *ids, const int64_t *offsets,
                       int64_t nlist, int d, const float *Q, int64_t nq, const int32_t *probes,
                       int nprobe, int kout, int64_t *out_ids, double *out_scores)
{
    if (!X || !ids || !offsets || !Q || !probes || !out_ids || !out_scores || d <= 0 ||
        nprobe <= 0 || kout <= 0 || dtype < 0 || dtype > 2)
        return -1;
    int err = 0;
#pragma omp parallel for schedule(dynamic)
    for (int64_t q = 0; q < nq; ++q) {
        int64_t total = 0;
        for (int r = 0; r < nprobe; ++r) {
            int32_t l = probes[q * nprobe + r];
            if (l < 0) continue;
            if (l >= nlist) { err = 2; l = -1; continue; }
            total += offsets[l + 1] - offsets[l];
        }
        cand_t *c = (cand_t *)malloc(sizeof(cand_t) * (size_t)(total > 0 ? total : 1));
        if (!c) { err = 1; continue; }
        int64_t m = 0;
        for (int r = 0; r < nprobe; ++r) {
            int32_t l = probes[q * nprobe + r];
            if (l < 0 || l >= nlist) continue;
            for (int64_t i = offsets[l]; i < offsets[l + 1]; ++i) {
                c[m].s = stored_dot(X, dtype, i, d, Q + q * d);
                c[m].id = ids[i];
                c[m].pos = i;
                ++m;
            }
        }
        qsort(c, (size_t)m, sizeof(cand_t), cand_cmp);
        for (int r = 0; r < kout; ++r) {
            if (r < m) {
                out_ids[q * kout + r] = c[r].id;
                out_scores[q * kout + r] = c[r].s;
            } else {
                out_ids[q * kout + r] = -1;
                out_scores[q * kout + r] = -INFINITY;
            }
        }
        free(c);
    }
    return err ? -2 : 0;
}

/* list[i] = arg-max_j <X_i, C_j> (fp64), ties -> smaller j; best[i] = that score (may be NULL) */
int oracle_assign(const void *X, int dtype, int64_t n, const float *C, int64_t nlist, int d,
                  int32_t *list, double *best)
{
    if (!X || !C || !list || nlist <= 0 || d <= 0 || (dtype != 0 && dtype != 1))
        return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double bs = -INFINITY;
        int64_t bj = 0;
        for (int64_t j = 0; j < nlist; ++j) {
            double s = 0.0;
            for (int t = 0; t < d; ++t)
                s += elem(X, dtype, i * d + t) * (double)C[j * d + t];
            if (s > bs) { bs = s; bj = j; }
        }
        list[i] = (int32_t)bj;
        if (best) best[i] = bs;
    }
    return 0;
}
