// Backlog-aware batch-size choice for the retrieval worker (host arithmetic only).
// With n requests queued, serving them as k equal batches one after the other gives an
// average latency of (k+1)/2 * T(n/k) minus the mean arrival time, where T(B) = a * B^c
// is the profiled time of one batch (paper Section 4.4, Eq. 4-6); one batch beats k
// batches exactly when 2 k^c <= k+1 (Eq. 7).  T is fitted to measured (B, T) samples of
// ivf_search.  Exports the ivf_sched_* part of include/ivf.h.
#include <cmath>
#include <cstdint>

#include "../../include/ivf.h"

extern "C" {

int ivf_sched_fit(const double* batch_sizes, const double* times, int m, double* a, double* c) {
    if (!batch_sizes || !times || !a || !c || m < 1) return IVF_ERR_INVALID;
    double mx = 0.0, my = 0.0;
    for (int i = 0; i < m; ++i) {
        if (!(batch_sizes[i] > 0.0) || !(times[i] > 0.0)) return IVF_ERR_INVALID;
        mx += std::log(batch_sizes[i]);
        my += std::log(times[i]);
    }
    mx /= m;
    my /= m;
    double sxx = 0.0, sxy = 0.0;
    for (int i = 0; i < m; ++i) {
        const double dx = std::log(batch_sizes[i]) - mx;
        sxx += dx * dx;
        sxy += dx * (std::log(times[i]) - my);
    }
    *c = sxx > 0.0 ? sxy / sxx : 0.0;
    *a = std::exp(my - *c * mx);
    return IVF_OK;
}

double ivf_sched_batch_time(double a, double c, double batch_size) { return a * std::pow(batch_size, c); }

int ivf_sched_avg_latency(double a, double c, int64_t n, int64_t k, double mean_arrival, double* latency) {
    if (!latency || n < 1 || k < 1 || !(a > 0.0) || c < 0.0) return IVF_ERR_INVALID;
    *latency = 0.5 * (double)(k + 1) * ivf_sched_batch_time(a, c, (double)n / (double)k) - mean_arrival;
    return IVF_OK;
}

int ivf_sched_single_batch_is_best(double c, int64_t k) {
    if (k < 1 || c < 0.0) return IVF_ERR_INVALID;
    return 2.0 * std::pow((double)k, c) <= (double)(k + 1) ? 1 : 0;
}

int ivf_sched_choose(double a, double c, int64_t n, const int64_t* candidates, int m, double mean_arrival,
                     int64_t* best_batch, double* best_latency) {
    if (!candidates || !best_batch || m < 1 || n < 1 || !(a > 0.0) || c < 0.0) return IVF_ERR_INVALID;
    bool have = false;
    int64_t bb = 0;
    double bl = 0.0;
    for (int i = 0; i < m; ++i) {
        const int64_t B = candidates[i];
        if (B < 1) return IVF_ERR_INVALID;
        // Batches served in turn: every request of a batch waits until that batch is done.
        // Full batches of B first, then one batch with the r requests that are left (which
        // takes T(r)); with r = 0 this is Eq. 6, with B >= n Eq. 5.
        const int64_t full = B >= n ? 0 : n / B;
        const int64_t r = n - full * B;
        const double tB = ivf_sched_batch_time(a, c, (double)B);
        double now = 0.0, waited = 0.0;             // clock; sum over requests of completion times
        for (int64_t j = 0; j < full; ++j) {
            now += tB;
            waited += (double)B * now;
        }
        if (r > 0) {
            now += ivf_sched_batch_time(a, c, (double)r);
            waited += (double)r * now;
        }
        const double L = waited / (double)n - mean_arrival;
        if (!have || L < bl || (L == bl && B > bb)) {
            have = true;
            bb = B;
            bl = L;
        }
    }
    *best_batch = bb;
    if (best_latency) *best_latency = bl;
    return IVF_OK;
}

}  // extern "C"
