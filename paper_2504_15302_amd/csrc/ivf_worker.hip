// Retrieval worker: the retrieval half of a decoupled retrieve-then-generate pipeline
// (paper Section 4.1: requests wait in a retrieval queue, a retrieval worker forms
// batches on its own and puts the retrieved contexts into the queue of the generation
// worker).  One host thread drains a request queue into batches, keeps up to two of them
// on the GPU at once (ivf_search_queued: the front stages of a batch run under the scan
// of the batch before it); finished results wait in a context queue until the consumer
// takes them.  The
// batch size for the current backlog comes from the backlog-aware rule (Section 4.4),
// fed by the worker's own timings.  Exports the ivf_worker_* part of include/ivf.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <condition_variable>
#include <cstring>
#include <deque>
#include <mutex>
#include <thread>
#include <unordered_map>
#include <unordered_set>
#include <vector>

#include "../../include/ivf.h"

namespace {

struct Request {
    uint64_t ticket;
    std::vector<float> q;
};
struct Result {
    std::vector<int64_t> ids;
    std::vector<float> scores;
};

}  // namespace

struct ivf_worker {
    ivf_index* idx = nullptr;
    int device = 0, d = 0, nprobe = 0, k = 0, max_batch = 0;
    std::thread th;
    std::mutex mu;
    std::condition_variable cv_req, cv_res;
    std::deque<Request> requests;                       // retrieval queue
    std::unordered_map<uint64_t, Result> done;          // context queue
    std::unordered_set<uint64_t> outstanding;           // submitted and not yet taken
    uint64_t next_ticket = 1;
    bool stopping = false, failed = false;
    int fail_code = 0;
    // per batch size (power of two index): smoothed time of one search, in ms
    std::vector<double> t_ms;
    std::vector<int> t_n;
    ivf_worker_stats st = {};
    int64_t wanted_budget = -1;                         // asked for and not yet taken up
};

namespace {

// One batch on its way through the GPU: its own pinned buffers and an event, so that the
// next batch can be issued while this one is still being searched.  The search reads the
// queries from the pinned buffer (its first stream copies them to the device, so the copy
// does not queue behind the batch before on the worker's stream) and its final selection
// writes the rows straight into the pinned result buffers.  Every batch goes to the one
// stream of the worker: a process has four hardware queues, the queued search needs three
// for its own streams, and streams that share a queue run one after the other.
struct Slot {
    hipEvent_t done = nullptr;                    // results have landed
    float *hq = nullptr, *hs = nullptr;
    int64_t* hi = nullptr;
    std::vector<Request> batch;
    bool busy = false;
    std::chrono::steady_clock::time_point issued;
};

bool slot_init(Slot& s, size_t B, int d, int k) {
    return hipEventCreateWithFlags(&s.done, hipEventDisableTiming) == hipSuccess &&
           hipHostMalloc(reinterpret_cast<void**>(&s.hq), B * d * sizeof(float)) == hipSuccess &&
           hipHostMalloc(reinterpret_cast<void**>(&s.hs), B * k * sizeof(float)) == hipSuccess &&
           hipHostMalloc(reinterpret_cast<void**>(&s.hi), B * k * sizeof(int64_t)) == hipSuccess;
}

void slot_free(Slot& s) {
    if (s.done) (void)hipEventDestroy(s.done);
    if (s.hq) (void)hipHostFree(s.hq);
    if (s.hs) (void)hipHostFree(s.hs);
    if (s.hi) (void)hipHostFree(s.hi);
}

// Queues the search of the slot's batch on the worker's stream.
int slot_issue(ivf_worker* w, Slot& s, hipStream_t st) {
    const size_t nb = s.batch.size();
    for (size_t i = 0; i < nb; ++i) std::memcpy(s.hq + i * w->d, s.batch[i].q.data(), sizeof(float) * w->d);
    s.issued = std::chrono::steady_clock::now();
    int rc = ivf_search_queued(w->idx, s.hq, (int64_t)nb, w->nprobe, w->k, s.hi, s.hs, st, nullptr);
    if (rc) return rc;
    if (hipEventRecord(s.done, st) != hipSuccess) return IVF_ERR_HIP;
    s.busy = true;
    return 0;
}

void worker_loop(ivf_worker* w) {
    if (hipSetDevice(w->device) != hipSuccess) { std::lock_guard<std::mutex> g(w->mu); w->failed = true; w->fail_code = IVF_ERR_HIP; w->cv_res.notify_all(); return; }
    constexpr int kSlots = 2;                      // batches in flight
    Slot slots[kSlots];
    hipStream_t st = nullptr;
    bool ok = hipStreamCreateWithFlags(&st, hipStreamNonBlocking) == hipSuccess;
    for (int i = 0; ok && i < kSlots; ++i) ok = slot_init(slots[i], (size_t)w->max_batch, w->d, w->k);
    std::vector<int64_t> cands;
    for (int b = 1; b <= w->max_batch; b <<= 1) cands.push_back(b);
    if (cands.back() != w->max_batch) cands.push_back(w->max_batch);
    bool moving = false, started = false, finish = false;
    int64_t budget = -1;
    int head = 0, inflight = 0;                    // slots[head] is the oldest batch in flight
    auto last_done = std::chrono::steady_clock::now();
    int fail_rc = 0;
    while (ok) {
        {
            std::unique_lock<std::mutex> lk(w->mu);
            auto wake = [&] { return w->stopping || !w->requests.empty() || w->wanted_budget >= 0; };
            if (inflight == 0) {                   // nothing to collect: sleep until there is something to do
                if (moving) w->cv_req.wait_for(lk, std::chrono::milliseconds(1), wake);   // an idle worker keeps the change going
                else w->cv_req.wait(lk, wake);
            }
            if (w->wanted_budget >= 0) {
                budget = w->wanted_budget;
                w->wanted_budget = -1;
            }
            finish = w->stopping && w->requests.empty() && inflight == 0;
        }
        if (budget >= 0 || moving) {
            // budget changes run beside the searches: start one between two batches, then
            // let every pass through the loop (and every search) carry it on
            int brc = 0;
            if (budget >= 0) {
                brc = ivf_set_device_budget_async(w->idx, budget);
                budget = -1;
                started = true;
            }
            int64_t pl = 0, pb = 0;
            int busy = 0;
            if (!brc && finish) brc = ivf_budget_wait(w->idx);      // nothing left to serve: see the change through
            if (!brc) brc = ivf_budget_progress(w->idx, &pl, &pb, &busy);
            ivf_info info;
            const bool have_info = ivf_get_info(w->idx, &info) == 0;
            moving = !brc && busy != 0;
            std::lock_guard<std::mutex> g(w->mu);
            if (started) { w->st.budget_changes += 1; started = false; }
            w->st.budget_pending_lists = brc ? 0 : pl;
            w->st.budget_busy = (moving || w->wanted_budget >= 0) ? 1 : 0;
            w->st.budget_error = brc;
            if (have_info) w->st.resident_lists = info.resident_lists;
        }
        // issue a batch if there are requests and a free slot
        bool issued = false;
        if (inflight < kSlots) {
            Slot& s = slots[(head + inflight) % kSlots];
            s.batch.clear();
            {
                std::unique_lock<std::mutex> lk(w->mu);
                if (!w->requests.empty()) {
                    const int64_t n = (int64_t)w->requests.size();
                    // batch size for this backlog: the backlog-aware rule once two batch sizes have
                    // been timed, the whole backlog (up to max_batch) before that
                    int64_t take = std::min<int64_t>(n, w->max_batch);
                    std::vector<double> bs, ts;
                    for (size_t i = 0; i < cands.size(); ++i)
                        if (w->t_n[i] > 0) { bs.push_back((double)cands[i]); ts.push_back(w->t_ms[i]); }
                    if (bs.size() >= 2) {
                        double a = 0, c = 0;
                        if (ivf_sched_fit(bs.data(), ts.data(), (int)bs.size(), &a, &c) == 0 && a > 0 && c >= 0) {
                            int64_t best = take;
                            if (ivf_sched_choose(a, c, n, cands.data(), (int)cands.size(), 0.0, &best, nullptr) == 0)
                                take = std::min<int64_t>(std::min<int64_t>(best, n), w->max_batch);
                            w->st.fit_a_ms = a;
                            w->st.fit_c = c;
                        }
                    }
                    for (int64_t i = 0; i < take; ++i) {
                        s.batch.push_back(std::move(w->requests.front()));
                        w->requests.pop_front();
                    }
                } else if (inflight == 0 && w->stopping && !moving && w->wanted_budget < 0) {
                    break;                                          // stopping and drained
                }
            }
            if (!s.batch.empty()) {
                if ((fail_rc = slot_issue(w, s, st))) break;
                inflight += 1;
                issued = true;
            }
        }
        // collect the oldest batch when nothing new could be issued (both slots taken, or no
        // request waiting): its service time runs from the later of its issue and the
        // completion of the batch before it
        if (inflight > 0 && !issued) {
            Slot& s = slots[head];
            if (hipEventSynchronize(s.done) != hipSuccess) { fail_rc = IVF_ERR_HIP; break; }
            const auto now = std::chrono::steady_clock::now();
            const double ms = std::chrono::duration<double, std::milli>(now - std::max(s.issued, last_done)).count();
            last_done = now;
            const size_t nb = s.batch.size();
            std::lock_guard<std::mutex> g(w->mu);
            for (size_t i = 0; i < nb; ++i) {
                Result r;
                r.ids.assign(s.hi + i * w->k, s.hi + (i + 1) * w->k);
                r.scores.assign(s.hs + i * w->k, s.hs + (i + 1) * w->k);
                w->done.emplace(s.batch[i].ticket, std::move(r));
            }
            // time of a batch of this size, filed under the smallest candidate that holds it
            size_t slot = 0;
            while (slot + 1 < cands.size() && (int64_t)nb > cands[slot]) ++slot;
            w->t_ms[slot] = w->t_n[slot] ? 0.75 * w->t_ms[slot] + 0.25 * ms : ms;
            w->t_n[slot] += 1;
            w->st.batches += 1;
            w->st.requests_done += (int64_t)nb;
            w->st.largest_batch = std::max<int64_t>(w->st.largest_batch, (int64_t)nb);
            w->cv_res.notify_all();
            s.busy = false;
            head = (head + 1) % kSlots;
            inflight -= 1;
        }
    }
    if (!ok || fail_rc) {
        std::lock_guard<std::mutex> g(w->mu);
        w->failed = true;
        w->fail_code = fail_rc ? fail_rc : IVF_ERR_OOM_DEVICE;
        w->cv_res.notify_all();
    }
    (void)hipGetLastError();
    if (st) { (void)hipStreamSynchronize(st); (void)hipStreamDestroy(st); }
    for (int i = 0; i < kSlots; ++i) slot_free(slots[i]);
}

}  // namespace

extern "C" {

int ivf_worker_start(ivf_index* idx, int nprobe, int k, int max_batch, ivf_worker** out) {
    if (!out) return IVF_ERR_INVALID;
    *out = nullptr;
    ivf_info info;
    if (!idx || ivf_get_info(idx, &info) != 0) return IVF_ERR_INVALID;
    if (nprobe < 1 || k < 1 || k > 1024 || max_batch < 1 || max_batch > 65535) return IVF_ERR_INVALID;
    ivf_worker* w = new (std::nothrow) ivf_worker();
    if (!w) return IVF_ERR_OOM_HOST;
    w->idx = idx; w->d = info.d; w->nprobe = nprobe; w->k = k; w->max_batch = max_batch;
    if (hipGetDevice(&w->device) != hipSuccess) { delete w; return IVF_ERR_HIP; }
    int nc = 0;
    for (int b = 1; b <= max_batch; b <<= 1) ++nc;
    w->t_ms.assign((size_t)nc + 1, 0.0);
    w->t_n.assign((size_t)nc + 1, 0);
    w->th = std::thread(worker_loop, w);
    *out = w;
    return 0;
}

int ivf_worker_submit(ivf_worker* w, const float* query, uint64_t* ticket) {
    if (!w || !query || !ticket) return IVF_ERR_INVALID;
    Request r;
    r.q.assign(query, query + w->d);
    std::lock_guard<std::mutex> g(w->mu);
    if (w->stopping) return IVF_ERR_INVALID;
    if (w->failed) return w->fail_code;
    r.ticket = w->next_ticket++;
    *ticket = r.ticket;
    w->outstanding.insert(r.ticket);
    w->requests.push_back(std::move(r));
    w->st.requests_submitted += 1;
    w->cv_req.notify_one();
    return 0;
}

int ivf_worker_wait(ivf_worker* w, uint64_t ticket, int64_t* out_ids, float* out_scores, int timeout_ms) {
    if (!w || !out_ids || !out_scores) return IVF_ERR_INVALID;
    std::unique_lock<std::mutex> lk(w->mu);
    if (!w->outstanding.count(ticket)) return IVF_ERR_INVALID;     // never issued, or taken before
    auto ready = [&] { return w->failed || w->done.count(ticket) != 0; };
    if (timeout_ms < 0) w->cv_res.wait(lk, ready);
    else if (!w->cv_res.wait_for(lk, std::chrono::milliseconds(timeout_ms), ready)) return 1;   // not ready yet
    auto it = w->done.find(ticket);
    if (it == w->done.end()) return w->failed ? w->fail_code : IVF_ERR_INVALID;   // failed, or taken before
    std::memcpy(out_ids, it->second.ids.data(), sizeof(int64_t) * w->k);
    std::memcpy(out_scores, it->second.scores.data(), sizeof(float) * w->k);
    w->done.erase(it);
    w->outstanding.erase(ticket);
    return 0;
}

int ivf_worker_get_stats(ivf_worker* w, ivf_worker_stats* out) {
    if (!w || !out) return IVF_ERR_INVALID;
    std::lock_guard<std::mutex> g(w->mu);
    *out = w->st;
    out->queued = (int64_t)w->requests.size();
    out->results_waiting = (int64_t)w->done.size();
    return 0;
}

int ivf_worker_set_device_budget(ivf_worker* w, int64_t bytes) {
    if (!w || bytes < 0) return IVF_ERR_INVALID;
    std::lock_guard<std::mutex> g(w->mu);
    if (w->stopping) return IVF_ERR_INVALID;
    if (w->failed) return w->fail_code;
    w->wanted_budget = bytes;
    w->st.budget_busy = 1;
    w->cv_req.notify_one();
    return 0;
}

int ivf_worker_stop(ivf_worker* w) {
    if (!w) return IVF_ERR_INVALID;
    {
        std::lock_guard<std::mutex> g(w->mu);
        w->stopping = true;
        w->cv_req.notify_all();
    }
    if (w->th.joinable()) w->th.join();
    const int rc = w->failed ? w->fail_code : 0;
    delete w;
    return rc;
}

}  // extern "C"
