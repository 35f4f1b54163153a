// Host-side bookkeeping of where list data lives.  Plain C++ (no HIP): the memory itself
// comes from two callbacks, so the same code manages HBM segments, pinned host segments,
// and — in the CPU tests — ordinary heap memory.
//
// List data lives in pools of fixed-size segments (one allocation each), carved in units
// of one 64-vector block.  A list is contiguous inside one segment.  Segments let a change
// of the device budget move only the lists that change tier and hand memory back segment
// by segment, without ever holding a second copy of a tier (the resident share of the
// vector database is adjusted at run time: paper Section 4.2 "Database partitions").
#pragma once
#include <algorithm>
#include <cstddef>
#include <cstdint>
#include <iterator>
#include <map>
#include <numeric>
#include <vector>

namespace ivf {

struct Seg {
    char* base = nullptr;
    size_t blocks = 0, used = 0;
    std::map<size_t, size_t> free;   // offset -> length, in blocks, coalesced
};

struct Pool {
    void* (*alloc)(size_t bytes) = nullptr;   // returns nullptr when out of memory
    void (*dealloc)(void* p) = nullptr;
    size_t block_bytes = 0, seg_blocks = 0;
    std::vector<Seg> segs;           // a dropped segment keeps its slot (base == nullptr)
    size_t allocated_blocks() const {
        size_t n = 0;
        for (const Seg& g : segs) n += g.blocks;
        return n;
    }
};

struct Loc {
    int8_t tier = 0;                 // 0 = HBM, 1 = pinned host
    int32_t seg = -1;                // -1: the list is empty
    size_t off = 0;                  // in blocks
};

inline void pool_free_all(Pool& p) {
    for (Seg& g : p.segs)
        if (g.base) p.dealloc(g.base);
    p.segs.clear();
}

// New segment of `blocks` blocks; returns its index or -1 when the allocation fails.
inline int pool_new_seg(Pool& p, size_t blocks) {
    char* base = static_cast<char*>(p.alloc(blocks * p.block_bytes));
    if (!base) return -1;
    int idx = -1;
    for (size_t i = 0; i < p.segs.size(); ++i)
        if (!p.segs[i].base) { idx = (int)i; break; }
    if (idx < 0) { p.segs.emplace_back(); idx = (int)p.segs.size() - 1; }
    Seg& g = p.segs[idx];
    g.base = base; g.blocks = blocks; g.used = 0;
    g.free.clear();
    g.free[0] = blocks;
    return idx;
}

// First fit over the existing segments (skipping `exclude`), then a new segment if allowed.
inline bool pool_alloc(Pool& p, size_t n, int& seg, size_t& off, bool may_grow, int exclude = -1) {
    for (size_t i = 0; i < p.segs.size(); ++i) {
        Seg& g = p.segs[i];
        if (!g.base || (int)i == exclude || g.blocks - g.used < n) continue;
        for (auto it = g.free.begin(); it != g.free.end(); ++it) {
            if (it->second < n) continue;
            const size_t o = it->first, len = it->second;
            g.free.erase(it);
            if (len > n) g.free[o + n] = len - n;
            g.used += n;
            seg = (int)i; off = o;
            return true;
        }
    }
    if (!may_grow) return false;
    int idx = pool_new_seg(p, std::max(p.seg_blocks, n));
    if (idx < 0 && p.seg_blocks > n) idx = pool_new_seg(p, n);
    if (idx < 0) return false;
    Seg& g = p.segs[idx];
    g.free.clear();
    if (g.blocks > n) g.free[n] = g.blocks - n;
    g.used = n;
    seg = idx; off = 0;
    return true;
}

inline void pool_release(Pool& p, int seg, size_t off, size_t n) {
    Seg& g = p.segs[seg];
    auto it = g.free.emplace(off, n).first;
    auto nx = std::next(it);
    if (nx != g.free.end() && it->first + it->second == nx->first) {
        it->second += nx->second;
        g.free.erase(nx);
    }
    if (it != g.free.begin()) {
        auto pv = std::prev(it);
        if (pv->first + pv->second == it->first) {
            pv->second += it->second;
            g.free.erase(it);
        }
    }
    g.used -= n;
}

inline void pool_drop_empty(Pool& p) {
    for (Seg& g : p.segs)
        if (g.base && g.used == 0) {
            p.dealloc(g.base);
            g = Seg();
        }
}

// Lists ranked by how much they deserve the fast tier: by lifetime probe count if `hits`
// is given (the "most probed first" policy), then by length, then by list number.
inline std::vector<int32_t> residency_order(const std::vector<int32_t>& len, const uint32_t* hits) {
    std::vector<int32_t> order(len.size());
    std::iota(order.begin(), order.end(), 0);
    std::sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
        if (hits && hits[a] != hits[b]) return hits[a] > hits[b];
        if (len[a] != len[b]) return len[a] > len[b];
        return a < b;
    });
    return order;
}

// res[l] = 1 for the lists that stay in (or come into) the fast tier under a budget of
// `bytes`: in rank order, while their padded size still fits; the first list that does
// not fit ends the selection.
inline std::vector<char> residency_choice(const std::vector<int32_t>& order, const std::vector<int32_t>& nblk,
                                          size_t block_bytes, uint64_t bytes) {
    std::vector<char> res(order.size(), 0);
    uint64_t used = 0;
    for (int32_t l : order) {
        const uint64_t b = (uint64_t)nblk[l] * block_bytes;
        if (used + b > bytes) break;
        used += b;
        res[l] = 1;
    }
    return res;
}

}  // namespace ivf
