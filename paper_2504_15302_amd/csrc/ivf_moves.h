// Where list data lives and how it moves between HBM and pinned host memory: the address
// table of the lists, and budget changes carried out as a background activity beside the
// searches (paper Section 4.2 "Database partitions"; Section 5 "Lazy dynamic transfer").
// Included by ivf_api.hip only.
#pragma once
#include "ivf_host.h"

namespace {

// Where list l is read from, as the host sees it (dev_ptr / host_ptr) and as the device
// table will see it (h_list_ptr: a host-resident list has a null entry, or — when the scan
// is to read pinned host memory directly — its host address tagged in bit 0).
void set_list_entry(ivf_index* x, int64_t l) {
    const Loc& c = x->loc[l];
    x->dev_ptr[l] = x->host_ptr[l] = nullptr;
    if (c.seg < 0) {         // empty list: a non-null device address marks it resident
        if (c.tier == 0) x->dev_ptr[l] = reinterpret_cast<const char*>(x->d_centroids);
    } else {
        const Pool& p = c.tier == 0 ? x->dpool : x->hpool;
        const char* a = p.segs[c.seg].base + c.off * p.block_bytes;
        (c.tier == 0 ? x->dev_ptr : x->host_ptr)[l] = a;
    }
    const char* t = x->dev_ptr[l];
    if (!t && x->host_ptr[l] && x->opt_host_direct)
        t = reinterpret_cast<const char*>(reinterpret_cast<uintptr_t>(x->host_ptr[l]) | 1u);
    x->h_list_ptr[l] = t;
}

void refresh_list_ptrs(ivf_index* x) {
    for (int64_t l = 0; l < x->nlist; ++l) set_list_entry(x, l);
}

// Device table of list addresses, copied from its host mirror (synchronous).
int upload_list_ptr_table(ivf_index* x) {
    refresh_list_ptrs(x);
    HIP_TRY(hipMemcpy(x->d_list_ptr, x->h_list_ptr, sizeof(void*) * (size_t)x->nlist, hipMemcpyHostToDevice));
    return 0;
}

// Events and pinned table snapshots are recycled between budget changes.
hipEvent_t take_event(ivf_index* x) {
    if (!x->spare_events.empty()) {
        hipEvent_t e = x->spare_events.back();
        x->spare_events.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;
    }
    return e;
}

const void** take_table(ivf_index* x) {
    if (!x->spare_tables.empty()) {
        const void** t = x->spare_tables.back();
        x->spare_tables.pop_back();
        return t;
    }
    const void** t = nullptr;
    if (hipHostMalloc(reinterpret_cast<void**>(&t), sizeof(void*) * (size_t)x->nlist) != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;
    }
    return t;
}

// Forgets a budget change in progress.  Only for an idle device whose pools are about to be
// freed as a whole: nothing is released list by list.
void moves_reset(ivf_index* x) {
    for (MoveBatch& b : x->inflight)
        if (b.landed) x->spare_events.push_back(b.landed);
    for (Limbo& lb : x->limbo) {
        if (lb.after) x->spare_events.push_back(lb.after);
        if (lb.table) x->spare_tables.push_back(lb.table);
    }
    x->inflight.clear(); x->limbo.clear(); x->todo.clear(); x->to_load.clear(); x->seg_skip.clear();
    for (const void** t : x->spare_tables) (void)hipHostFree(t);   // sized for the index that goes away
    x->spare_tables.clear();
    x->phase = kPhaseIdle;
    x->inflight_bytes = 0;
    x->pending_lists = x->pending_bytes = 0;
    x->move_rc = 0;
    x->move_msg.clear();
    x->search_end_recorded = false;
}

// ---- budget changes as a background activity -------------------------------------------

bool moves_active(const ivf_index* x) {
    return x->phase != kPhaseIdle || !x->inflight.empty() || !x->limbo.empty();
}

char* loc_addr(ivf_index* x, const Loc& c) {
    Pool& p = c.tier == 0 ? x->dpool : x->hpool;
    return p.segs[c.seg].base + c.off * p.block_bytes;
}

void release_place(ivf_index* x, const Loc& c, int32_t l) {
    pool_release(c.tier == 0 ? x->dpool : x->hpool, c.seg, c.off, (size_t)x->nblk[l]);
}

// Ends a change early: what has not been issued is dropped (reserved places are handed
// back).  Copies already issued still land and are committed by moves_advance.
void moves_stop(ivf_index* x, int rc, const std::string& msg) {
    for (const Move& m : x->todo)
        if (m.placed) release_place(x, m.to, m.l);
    x->todo.clear();
    x->to_load.clear();
    x->phase = kPhaseIdle;
    if (rc) {
        x->move_rc = rc;
        x->move_msg = msg;
    }
}

// Sends the address table to the device behind the searches issued so far (the copy reads
// a snapshot, so a later change of the mirror cannot reach an earlier search) and parks
// the old places of `lb` until that has happened.
int push_table(ivf_index* x, Limbo& lb) {
    std::memcpy(lb.table, x->h_list_ptr, sizeof(void*) * (size_t)x->nlist);
    if (x->search_end_recorded) HIP_TRY(hipStreamWaitEvent(x->patch_stream, x->ev_search_end, 0));
    HIP_TRY(hipMemcpyAsync(x->d_list_ptr, lb.table, sizeof(void*) * (size_t)x->nlist, hipMemcpyHostToDevice, x->patch_stream));
    HIP_TRY(hipEventRecord(lb.after, x->patch_stream));
    x->limbo.push_back(std::move(lb));
    return 0;
}

// Compaction of the HBM pool: picks the least-filled segment whose lists fit into the
// holes of the other segments, reserves those holes and queues the device-to-device moves.
bool compact_pick(ivf_index* x) {
    Pool& p = x->dpool;
    std::vector<int> segs;
    size_t total_free = 0;
    for (size_t i = 0; i < p.segs.size(); ++i) {
        if (!p.segs[i].base) continue;
        total_free += p.segs[i].blocks - p.segs[i].used;
        if (p.segs[i].used > 0 && !(i < x->seg_skip.size() && x->seg_skip[i])) segs.push_back((int)i);
    }
    std::sort(segs.begin(), segs.end(), [&](int a, int b) { return p.segs[a].used < p.segs[b].used; });
    for (int sidx : segs) {
        const Seg& g = p.segs[sidx];
        if (total_free - (g.blocks - g.used) < g.used) continue;
        std::vector<int32_t> lists;
        for (int64_t l = 0; l < x->nlist; ++l)
            if (x->loc[l].tier == 0 && x->loc[l].seg == sidx) lists.push_back((int32_t)l);
        if (lists.empty()) continue;
        std::sort(lists.begin(), lists.end(), [&](int32_t a, int32_t b) {
            return x->nblk[a] != x->nblk[b] ? x->nblk[a] > x->nblk[b] : a < b;     // large lists first: first fit packs better
        });
        std::vector<Move> mv;
        bool ok = true;
        for (int32_t l : lists) {
            Move m;
            m.l = l; m.from = x->loc[l]; m.to.tier = 0; m.placed = true;
            if (!pool_alloc(p, (size_t)x->nblk[l], m.to.seg, m.to.off, false, sidx)) { ok = false; break; }
            mv.push_back(m);
        }
        if (!ok) {                                   // holes too small: leave this segment alone
            for (const Move& m : mv) release_place(x, m.to, m.l);
            if ((size_t)sidx < x->seg_skip.size()) x->seg_skip[sidx] = 1;
            continue;
        }
        for (const Move& m : mv) x->todo.push_back(m);
        return true;
    }
    return false;
}

// The current phase has nothing left to issue, in flight or in limbo: go on to the next.
void next_phase(ivf_index* x) {
    if (x->phase == kPhaseEvict) {
        x->phase = kPhaseCompact;
        x->seg_skip.assign(x->dpool.segs.size(), 0);
    }
    if (x->phase == kPhaseCompact) {
        pool_drop_empty(x->dpool);                   // the segment emptied last, if any
        if (x->compact_wanted && compact_pick(x)) return;
        x->phase = kPhaseLoad;
        for (int32_t l : x->to_load) {
            Move m;
            m.l = l; m.from = x->loc[l]; m.to.tier = 0;
            x->todo.push_back(m);
        }
        x->to_load.clear();
        if (!x->todo.empty()) return;
    }
    pool_drop_empty(x->hpool);
    x->phase = kPhaseIdle;
}

// One non-blocking step of the change in progress: releases old places whose readers are
// done, switches over the lists whose copies have landed, issues further copies.
int moves_advance(ivf_index* x) {
    while (!x->limbo.empty()) {
        Limbo& lb = x->limbo.front();
        hipError_t q = hipEventQuery(lb.after);
        if (q == hipErrorNotReady) { (void)hipGetLastError(); break; }
        if (q != hipSuccess) { (void)hipGetLastError(); return fail(IVF_ERR_HIP, "list table update failed: %s", hipGetErrorString(q)); }
        for (const Move& m : lb.moves) release_place(x, m.from, m.l);
        x->spare_events.push_back(lb.after);
        x->spare_tables.push_back(lb.table);
        x->limbo.pop_front();
    }
    {
        Limbo lb;
        while (!x->inflight.empty()) {
            MoveBatch& b = x->inflight.front();
            hipError_t q = hipEventQuery(b.landed);
            if (q == hipErrorNotReady) { (void)hipGetLastError(); break; }
            if (q != hipSuccess) { (void)hipGetLastError(); return fail(IVF_ERR_HIP, "moving lists failed: %s", hipGetErrorString(q)); }
            if (!lb.after) {
                lb.after = take_event(x);
                lb.table = take_table(x);
                if (!lb.after || !lb.table) {
                    if (lb.after) x->spare_events.push_back(lb.after);
                    if (lb.table) x->spare_tables.push_back(lb.table);
                    return fail(IVF_ERR_OOM_HOST, "no event or pinned table for a list table update");
                }
            }
            for (const Move& m : b.moves) {
                x->loc[m.l] = m.to;
                set_list_entry(x, m.l);
                const int64_t by = (int64_t)((size_t)x->nblk[m.l] * x->block_bytes);
                if (m.from.tier == 0 && m.to.tier == 1) { x->moved_d2h += by; x->resident_lists -= 1; }
                else if (m.from.tier == 1 && m.to.tier == 0) { x->moved_h2d += by; x->resident_lists += 1; }
                else x->moved_d2d += by;
                lb.moves.push_back(m);
            }
            x->inflight_bytes -= b.bytes;
            x->spare_events.push_back(b.landed);
            x->inflight.pop_front();
        }
        if (lb.after) {
            int rc = push_table(x, lb);
            if (rc) return rc;
        }
    }
    const size_t chunk = (size_t)x->opt_move_chunk_kb << 10, cap = (size_t)x->opt_move_inflight_kb << 10;
    while (x->phase != kPhaseIdle) {
        if (x->todo.empty()) {
            if (!x->inflight.empty() || !x->limbo.empty()) break;
            next_phase(x);
            continue;
        }
        if (x->inflight_bytes >= cap) break;
        MoveBatch b;
        b.landed = take_event(x);
        if (!b.landed) { moves_stop(x, IVF_ERR_HIP, "no event for a batch of list copies"); break; }
        while (!x->todo.empty() && b.bytes < chunk && x->inflight_bytes + b.bytes < cap) {
            Move m = x->todo.front();
            const size_t nb = (size_t)x->nblk[m.l];
            if (!m.placed && !pool_alloc(m.to.tier == 0 ? x->dpool : x->hpool, nb, m.to.seg, m.to.off, true)) {
                char msg[128];
                std::snprintf(msg, sizeof msg, "out of %s memory while moving list %d", m.to.tier == 0 ? "device" : "pinned host", m.l);
                moves_stop(x, m.to.tier == 0 ? IVF_ERR_OOM_DEVICE : IVF_ERR_OOM_HOST, msg);
                break;
            }
            x->todo.pop_front();
            hipError_t e = hipMemcpyAsync(loc_addr(x, m.to), loc_addr(x, m.from), nb * x->block_bytes, hipMemcpyDefault, x->move_stream);
            if (e != hipSuccess) {
                (void)hipGetLastError();
                release_place(x, m.to, m.l);
                moves_stop(x, IVF_ERR_HIP, std::string("copy of a list failed: ") + hipGetErrorString(e));
                break;
            }
            b.moves.push_back(m);
            b.bytes += nb * x->block_bytes;
        }
        if (b.moves.empty()) { x->spare_events.push_back(b.landed); break; }
        hipError_t e = hipEventRecord(b.landed, x->move_stream);
        if (e != hipSuccess) {
            // the copies cannot be tracked: wait for them here, the batch then counts as landed
            (void)hipGetLastError();
            (void)hipStreamSynchronize(x->move_stream);
            (void)hipEventRecord(b.landed, x->move_stream);
        }
        x->inflight_bytes += b.bytes;
        x->inflight.push_back(std::move(b));
    }
    return 0;
}

// Blocks until no change is in progress.  With `cancel`, what has not been issued is dropped.
int moves_drain(ivf_index* x, bool cancel) {
    if (cancel && x->phase != kPhaseIdle) moves_stop(x, 0, "");
    while (moves_active(x)) {
        int rc = moves_advance(x);
        if (rc) return rc;
        if (!x->inflight.empty()) HIP_TRY(hipEventSynchronize(x->inflight.front().landed));
        else if (!x->limbo.empty()) HIP_TRY(hipEventSynchronize(x->limbo.front().after));
    }
    return 0;
}

// Works out which lists have to change tier for a budget of `bytes` and queues the change.
// The device is idle and no change is in progress.
int budget_plan(ivf_index* x, int64_t bytes) {
    const int64_t nlist = x->nlist;
    int rc_streams = need_stream(x->move_stream);
    if (!rc_streams) rc_streams = need_stream(x->patch_stream);
    if (rc_streams) return rc_streams;
    x->moved_h2d = x->moved_d2h = x->moved_d2d = 0;
    x->move_rc = 0;
    x->move_msg.clear();
    x->search_end_recorded = false;
    // which lists are to be resident: ranked by the policy, while they fit
    std::vector<uint32_t> hits;
    if (x->opt_policy == 1) {
        hits.resize((size_t)nlist);
        HIP_TRY(hipMemcpy(hits.data(), x->d_hits, sizeof(uint32_t) * (size_t)nlist, hipMemcpyDeviceToHost));
    }
    const std::vector<int32_t> order = residency_order(x->len, hits.empty() ? nullptr : hits.data());
    const std::vector<char> res = residency_choice(order, x->nblk, x->block_bytes, (uint64_t)bytes);
    // evictions go least valuable first, loads most valuable first; a list without data
    // just changes its label
    bool relabelled = false;
    for (auto it = order.rbegin(); it != order.rend(); ++it) {
        const int32_t l = *it;
        if (x->loc[l].tier != 0 || res[l]) continue;
        if (x->nblk[l] == 0) { x->loc[l].tier = 1; x->resident_lists -= 1; relabelled = true; continue; }
        Move m;
        m.l = l; m.from = x->loc[l]; m.to.tier = 1;
        x->todo.push_back(m);
    }
    for (int32_t l : order) {
        if (x->loc[l].tier != 1 || !res[l]) continue;
        if (x->nblk[l] == 0) { x->loc[l].tier = 0; x->resident_lists += 1; relabelled = true; continue; }
        x->to_load.push_back(l);
    }
    if (relabelled) {
        int rc = upload_list_ptr_table(x);
        if (rc) return rc;
    }
    if (x->todo.empty() && x->to_load.empty()) return 0;
    x->compact_wanted = !x->todo.empty();
    x->phase = kPhaseEvict;
    return 0;
}

void count_pending(const ivf_index* x, int64_t& lists, int64_t& bytes) {
    lists = bytes = 0;
    auto add = [&](int32_t l) { lists += 1; bytes += (int64_t)((size_t)x->nblk[l] * x->block_bytes); };
    for (const MoveBatch& b : x->inflight)
        for (const Move& m : b.moves)
            if (m.from.tier != m.to.tier) add(m.l);
    for (const Move& m : x->todo)
        if (m.from.tier != m.to.tier) add(m.l);
    for (int32_t l : x->to_load) add(l);
}

}  // namespace
