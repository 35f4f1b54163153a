/*
 * A consumer of the C ABI written in plain C: builds a small IVF index from host arrays,
 * moves half of it to pinned host memory, searches a batch of queries and checks the
 * result against a brute-force scan of the probed lists done right here on the host.
 * Device memory for queries and results comes from the HIP runtime; nothing else is used.
 *
 *   hipcc -x c examples/search_demo.c ... is not needed: any C compiler will do, e.g.
 *   gcc -std=c99 -D__HIP_PLATFORM_AMD__ -I/opt/rocm/include -Iinclude examples/search_demo.c \
 *       -Lpaper_2504_15302_amd -livf_mi355x -L/opt/rocm/lib -lamdhip64 -lm -o search_demo
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "ivf.h"

#define D 32
#define NLIST 8
#define N 4000
#define NQ 5
#define NPROBE 3
#define K 4

static unsigned long long rng_state = 88172645463325252ull;
static float rnd(void) /* xorshift, uniform in [-1, 1) */
{
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return (float)((rng_state >> 11) % 2000001ull) / 1000000.0f - 1.0f;
}

static double dot(const float *a, const float *b)
{
    double s = 0;
    int t;
    for (t = 0; t < D; ++t) s += (double)a[t] * (double)b[t];
    return s;
}

#define CHECK_IVF(call)                                                          \
    do {                                                                         \
        int rc_ = (call);                                                        \
        if (rc_ != 0) {                                                          \
            fprintf(stderr, "%s -> %d: %s\n", #call, rc_, ivf_last_error());     \
            return 1;                                                            \
        }                                                                        \
    } while (0)
#define CHECK_HIP(call)                                                          \
    do {                                                                         \
        hipError_t e_ = (call);                                                  \
        if (e_ != hipSuccess) {                                                  \
            fprintf(stderr, "%s -> %s\n", #call, hipGetErrorString(e_));         \
            return 1;                                                            \
        }                                                                        \
    } while (0)

int main(void)
{
    static float cen[NLIST * D], raw[N * D], vec[N * D], q[NQ * D];
    static int label[N];
    static int64_t ids[N], off[NLIST + 1];
    int64_t h_ids[NQ * K];
    float h_scores[NQ * K];
    int i, j, t, r, bad = 0;

    for (i = 0; i < NLIST * D; ++i) cen[i] = rnd();
    for (i = 0; i < N * D; ++i) raw[i] = rnd();
    for (i = 0; i < NQ * D; ++i) q[i] = rnd();
    /* list of a vector = centroid with the largest inner product; vectors grouped by list */
    memset(off, 0, sizeof off);
    for (i = 0; i < N; ++i) {
        double best = -1e300;
        for (j = 0; j < NLIST; ++j) {
            double s = dot(raw + i * D, cen + j * D);
            if (s > best) { best = s; label[i] = j; }
        }
        off[label[i] + 1] += 1;
    }
    for (j = 0; j < NLIST; ++j) off[j + 1] += off[j];
    {
        int64_t cursor[NLIST];
        for (j = 0; j < NLIST; ++j) cursor[j] = off[j];
        for (i = 0; i < N; ++i) {
            int64_t p = cursor[label[i]]++;
            memcpy(vec + p * D, raw + i * D, sizeof(float) * D);
            ids[p] = 1000 + 3 * (int64_t)i;            /* user ids: anything unique */
        }
    }

    ivf_index *idx = NULL;
    CHECK_IVF(ivf_index_create(&idx));
    CHECK_IVF(ivf_index_upload(idx, D, NLIST, N, cen, vec, IVF_FP32, ids, off));
    {
        ivf_info info;
        CHECK_IVF(ivf_get_info(idx, &info));
        CHECK_IVF(ivf_set_device_budget(idx, info.index_bytes / 2));
        CHECK_IVF(ivf_get_info(idx, &info));
        printf("index: %lld vectors, %lld lists, %lld of them in HBM, %lld bytes in pinned host memory\n",
               (long long)info.n, (long long)info.nlist, (long long)info.resident_lists,
               (long long)info.host_list_bytes);
    }

    float *d_q = NULL, *d_scores = NULL;
    int64_t *d_ids = NULL;
    CHECK_HIP(hipMalloc((void **)&d_q, sizeof q));
    CHECK_HIP(hipMalloc((void **)&d_ids, sizeof h_ids));
    CHECK_HIP(hipMalloc((void **)&d_scores, sizeof h_scores));
    CHECK_HIP(hipMemcpy(d_q, q, sizeof q, hipMemcpyHostToDevice));
    CHECK_IVF(ivf_search(idx, d_q, NQ, NPROBE, K, d_ids, d_scores, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_HIP(hipMemcpy(h_ids, d_ids, sizeof h_ids, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(h_scores, d_scores, sizeof h_scores, hipMemcpyDeviceToHost));

    /* the same on the host: the NPROBE best centroids, then every vector of those lists */
    for (r = 0; r < NQ; ++r) {
        int probe[NPROBE];
        double cs[NLIST];
        for (j = 0; j < NLIST; ++j) cs[j] = dot(q + r * D, cen + j * D);
        for (t = 0; t < NPROBE; ++t) {
            int bj = -1;
            for (j = 0; j < NLIST; ++j) {
                int taken = 0, u;
                for (u = 0; u < t; ++u) taken |= probe[u] == j;
                if (!taken && (bj < 0 || cs[j] > cs[bj])) bj = j;
            }
            probe[t] = bj;
        }
        for (t = 0; t < K; ++t) {           /* t-th best candidate by (score desc, id asc) */
            double bs = -1e300;
            int64_t bid = -1;
            int u;
            for (u = 0; u < NPROBE; ++u) {
                int64_t p;
                for (p = off[probe[u]]; p < off[probe[u] + 1]; ++p) {
                    double s = dot(q + r * D, vec + p * D);
                    int used = 0, v;
                    for (v = 0; v < t; ++v) used |= h_ids[r * K + v] == ids[p];
                    if (!used && (s > bs || (s == bs && ids[p] < bid))) { bs = s; bid = ids[p]; }
                }
            }
            if (h_ids[r * K + t] != bid || fabs((double)h_scores[r * K + t] - bs) > 1e-5 * fabs(bs)) {
                printf("query %d rank %d: library (%lld, %.6f), host (%lld, %.6f)\n", r, t,
                       (long long)h_ids[r * K + t], h_scores[r * K + t], (long long)bid, bs);
                bad = 1;
            }
        }
        printf("query %d: best chunk %lld (score %.4f)\n", r, (long long)h_ids[r * K], h_scores[r * K]);
    }
    (void)hipFree(d_q);
    (void)hipFree(d_ids);
    (void)hipFree(d_scores);
    ivf_index_destroy(idx);
    printf(bad ? "MISMATCH\n" : "ok\n");
    return bad;
}
