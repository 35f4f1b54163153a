// CPU test of the list-pool bookkeeping (paper_2504_15302_amd/csrc/ivf_pool.h) against a
// byte map kept by the test: random allocations and releases over heap memory standing in
// for HBM / pinned segments.  Prints "ok" and returns 0, or says what broke.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <set>
#include <vector>

#include "../../paper_2504_15302_amd/csrc/ivf_pool.h"

using namespace ivf;

static size_t g_live_allocs = 0, g_fail_after = (size_t)-1;
static void* test_alloc(size_t bytes) {
    if (g_fail_after == 0) return nullptr;
    if (g_fail_after != (size_t)-1) --g_fail_after;
    ++g_live_allocs;
    return std::malloc(bytes ? bytes : 1);
}
static void test_free(void* p) {
    --g_live_allocs;
    std::free(p);
}

#define CHECK(cond, ...)                                     \
    do {                                                     \
        if (!(cond)) {                                       \
            std::printf("FAILED %s:%d: ", __FILE__, __LINE__); \
            std::printf(__VA_ARGS__);                        \
            std::printf("\n");                               \
            return 1;                                        \
        }                                                    \
    } while (0)

struct Held { int seg; size_t off, n; unsigned char tag; };

// every invariant of a pool, given the allocations the test believes are live
static int check_pool(const Pool& p, const std::vector<Held>& held) {
    std::vector<std::vector<char>> map(p.segs.size());
    for (size_t i = 0; i < p.segs.size(); ++i) map[i].assign(p.segs[i].blocks, 0);
    std::vector<size_t> used(p.segs.size(), 0);
    for (const Held& h : held) {
        CHECK(h.seg >= 0 && (size_t)h.seg < p.segs.size() && p.segs[h.seg].base, "allocation in a dropped segment");
        CHECK(h.off + h.n <= p.segs[h.seg].blocks, "allocation past the end of its segment");
        for (size_t b = h.off; b < h.off + h.n; ++b) {
            CHECK(!map[h.seg][b], "two allocations overlap in segment %d block %zu", h.seg, b);
            map[h.seg][b] = 1;
        }
        used[h.seg] += h.n;
        // the bytes written at allocation time are still there
        const unsigned char* a = reinterpret_cast<const unsigned char*>(p.segs[h.seg].base) + h.off * p.block_bytes;
        for (size_t i = 0; i < h.n * p.block_bytes; i += 97) CHECK(a[i] == h.tag, "memory of a live allocation was overwritten");
    }
    for (size_t i = 0; i < p.segs.size(); ++i) {
        const Seg& g = p.segs[i];
        if (!g.base) { CHECK(g.blocks == 0 && g.used == 0 && g.free.empty(), "dropped segment keeps state"); continue; }
        CHECK(g.used == used[i], "segment %zu: used %zu, live allocations %zu", i, g.used, used[i]);
        size_t free_blocks = 0, prev_end = (size_t)-1;
        for (const auto& f : g.free) {
            CHECK(f.second > 0 && f.first + f.second <= g.blocks, "bad free range");
            CHECK(prev_end == (size_t)-1 || f.first > prev_end, "free ranges not coalesced or out of order");
            for (size_t b = f.first; b < f.first + f.second; ++b) CHECK(!map[i][b], "free range covers a live block");
            free_blocks += f.second;
            prev_end = f.first + f.second;
        }
        CHECK(free_blocks + g.used == g.blocks, "segment %zu: free %zu + used %zu != %zu", i, free_blocks, g.used, g.blocks);
    }
    return 0;
}

static int random_walk(unsigned seed, size_t seg_blocks, size_t max_n) {
    std::mt19937 rng(seed);
    Pool p;
    p.alloc = test_alloc; p.dealloc = test_free;
    p.block_bytes = 64; p.seg_blocks = seg_blocks;
    std::vector<Held> held;
    unsigned char tag = 1;
    for (int step = 0; step < 4000; ++step) {
        const int op = (int)(rng() % 100);
        if (op < 55 || held.empty()) {
            const size_t n = 1 + rng() % max_n;
            const bool grow = rng() % 4 != 0;
            int exclude = (rng() % 5 == 0 && !p.segs.empty()) ? (int)(rng() % p.segs.size()) : -1;
            if (exclude >= 0 && !p.segs[exclude].base) exclude = -1;      // only a live segment can be excluded
            // would first fit find room without growing?
            bool room = false;
            for (size_t i = 0; i < p.segs.size() && !room; ++i) {
                if (!p.segs[i].base || (int)i == exclude) continue;
                for (const auto& f : p.segs[i].free) if (f.second >= n) { room = true; break; }
            }
            Held h{-1, 0, n, tag};
            const bool ok = pool_alloc(p, n, h.seg, h.off, grow, exclude);
            CHECK(ok == (room || grow), "alloc of %zu blocks: got %d, room %d, grow %d", n, (int)ok, (int)room, (int)grow);
            if (ok) {
                CHECK(h.seg != exclude, "allocation landed in the excluded segment");
                std::memset(p.segs[h.seg].base + h.off * p.block_bytes, tag, n * p.block_bytes);
                held.push_back(h);
                tag = (unsigned char)(tag % 250 + 1);
            }
        } else if (op < 95) {
            const size_t i = rng() % held.size();
            pool_release(p, held[i].seg, held[i].off, held[i].n);
            held[i] = held.back();
            held.pop_back();
        } else {
            const size_t before = g_live_allocs;
            size_t empty = 0;
            for (const Seg& g : p.segs) empty += g.base && g.used == 0;
            pool_drop_empty(p);
            CHECK(before - g_live_allocs == empty, "drop_empty freed %zu segments, %zu were empty", before - g_live_allocs, empty);
        }
        if (step % 50 == 0 && check_pool(p, held)) return 1;
    }
    if (check_pool(p, held)) return 1;
    for (const Held& h : held) pool_release(p, h.seg, h.off, h.n);
    held.clear();
    if (check_pool(p, held)) return 1;
    for (const Seg& g : p.segs)
        if (g.base) CHECK(g.free.size() == 1 && g.free.begin()->second == g.blocks, "an empty segment is not one free range");
    pool_free_all(p);
    CHECK(g_live_allocs == 0, "%zu segments leaked", g_live_allocs);
    return 0;
}

static int out_of_memory() {
    Pool p;
    p.alloc = test_alloc; p.dealloc = test_free;
    p.block_bytes = 16; p.seg_blocks = 100;
    int seg; size_t off;
    g_fail_after = 1;                                   // one segment, then nothing
    CHECK(pool_alloc(p, 60, seg, off, true), "first allocation");
    CHECK(!pool_alloc(p, 60, seg, off, true), "second allocation must fail: no room, no memory");
    CHECK(pool_alloc(p, 40, seg, off, true) && off == 60, "the rest of the first segment is still usable");
    g_fail_after = (size_t)-1;
    // a request larger than a segment gets a segment of its own size
    CHECK(pool_alloc(p, 250, seg, off, true) && p.segs[seg].blocks == 250 && off == 0, "oversized request");
    pool_free_all(p);
    CHECK(g_live_allocs == 0, "leak");
    return 0;
}

static int residency() {
    // lengths with ties, an empty list, probe counts that disagree with the lengths
    const std::vector<int32_t> len = {100, 300, 300, 0, 64, 65, 1000};
    std::vector<int32_t> nblk;
    for (int32_t l : len) nblk.push_back((l + 63) / 64);
    const std::vector<int32_t> by_len = residency_order(len, nullptr);
    const std::vector<int32_t> want_len = {6, 1, 2, 0, 5, 4, 3};
    CHECK(by_len == want_len, "ranking by length (ties to the smaller list)");
    const std::vector<uint32_t> hits = {5, 0, 9, 9, 0, 5, 0};
    const std::vector<int32_t> by_hits = residency_order(len, hits.data());
    const std::vector<int32_t> want_hits = {2, 3, 0, 5, 6, 1, 4};
    CHECK(by_hits == want_hits, "ranking by probe count, then length, then number");
    const size_t bb = 10;
    // blocks: 2 5 5 0 1 2 16; by length: 16, 5, 5, 2, 2, 1, 0
    std::vector<char> r = residency_choice(by_len, nblk, bb, 16 * bb + 5 * bb + 4 * bb);
    CHECK((r == std::vector<char>{0, 1, 0, 0, 0, 0, 1}), "selection stops at the first list that does not fit");
    r = residency_choice(by_len, nblk, bb, 0);
    CHECK((r == std::vector<char>{0, 0, 0, 0, 0, 0, 0}), "zero budget keeps nothing (the empty list ranks last)");
    r = residency_choice(by_len, nblk, bb, 31 * bb);
    CHECK((r == std::vector<char>{1, 1, 1, 1, 1, 1, 1}), "a budget of the whole index keeps everything");
    r = residency_choice(by_hits, nblk, bb, 5 * bb);
    CHECK((r == std::vector<char>{0, 0, 1, 1, 0, 0, 0}), "most probed first, the empty list costs nothing");
    return 0;
}

int main() {
    for (unsigned seed = 1; seed <= 6; ++seed)
        if (random_walk(seed, seed % 2 ? 64 : 500, seed % 3 ? 20 : 90)) return 1;
    if (out_of_memory()) return 1;
    if (residency()) return 1;
    std::printf("ok\n");
    return 0;
}
