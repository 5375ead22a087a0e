// Test-only: the library's host-side code (block pool, host arena, residency index, forecaster, the
// scheduling arithmetic) driven hard in a plain executable, to be built with AddressSanitizer +
// UBSan, and again with ThreadSanitizer.  It checks its own invariants and prints "ok".
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <set>
#include <thread>
#include <vector>

#include "tc_blocks.h"
#include "tc_map.h"
#include "tokencake_kv.h"

#define REQUIRE(c) do { if (!(c)) { std::printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #c); std::exit(1); } } while (0)

static void block_pool_stream(uint32_t seed)
{
    std::mt19937 rng(seed);
    const uint32_t NB = 97;
    tc::BlockPool bp(NB);
    std::vector<std::vector<int32_t>> held, flying;
    std::vector<int> owned(NB, 0);
    for (int step = 0; step < 20000; ++step) {
        const uint32_t r = rng() % 100;
        if (r < 30) {
            uint32_t n = rng() % 12;
            std::vector<int32_t> out(n ? n : 1);
            if (bp.alloc(n, out.data()) == TC_OK) {
                out.resize(n);
                for (int32_t b : out) { REQUIRE(b >= 0 && uint32_t(b) < NB && owned[b] == 0); owned[b] = 1; }
                if (n) held.push_back(out);
            }
        } else if (r < 45) {
            uint32_t n = rng() % 8;
            std::vector<int32_t> pref(n ? n : 1), out(n ? n : 1);
            for (uint32_t i = 0; i < n; ++i) pref[i] = int32_t(rng() % (NB + 4)) - 2;
            if (bp.alloc_prefer(pref.data(), n, out.data()) == TC_OK) {
                out.resize(n);
                for (int32_t b : out) { REQUIRE(b >= 0 && uint32_t(b) < NB && owned[b] == 0); owned[b] = 1; }
                if (n) held.push_back(out);
            }
        } else if (r < 55 && !held.empty()) {
            auto &ids = held[rng() % held.size()];
            REQUIRE(bp.ref(ids.data(), uint32_t(ids.size())) == TC_OK);
            for (int32_t b : ids) ++owned[b];
            held.push_back(ids);
        } else if (r < 80 && !held.empty()) {
            size_t k = rng() % held.size();
            std::vector<int32_t> ids = held[k];
            held.erase(held.begin() + long(k));
            if (rng() % 2 && bp.check_transfer(ids.data(), uint32_t(ids.size())) == TC_OK) {
                bp.begin_transfer(ids.data(), uint32_t(ids.size()));
                flying.push_back(ids);
            }
            REQUIRE(bp.free(ids.data(), uint32_t(ids.size())) == TC_OK);
            for (int32_t b : ids) --owned[b];
        } else if (r < 92 && !flying.empty()) {
            bp.end_transfer(flying.front().data(), uint32_t(flying.front().size()));
            flying.erase(flying.begin());
        } else {
            int32_t bad[3] = {int32_t(rng() % NB), -1, int32_t(NB)};
            REQUIRE(bp.free(bad + 1, 1) == TC_ERR_RANGE && bp.ref(bad + 2, 1) == TC_ERR_RANGE);
            int32_t twice[2] = {bad[0], bad[0]};
            REQUIRE(bp.alloc_at(twice, 2) != TC_OK);
        }
        REQUIRE(bp.n_free() + bp.n_used() + bp.n_pending() == NB);
    }
}

// The work-item arithmetic of the copy kernels, walked on the CPU exactly as a launch walks it: every
// item is taken once and only once, by a workgroup of the right run, and nothing outside [0, n_items).
static void item_mapping(uint32_t seed)
{
    std::mt19937 rng(seed);
    // division by multiplication: exact for every n < 2^31
    const uint32_t divisors[] = {1, 2, 3, 5, 7, 8, 10, 64, 96, 127, 128, 160, 255, 256, 1000, 65535, 65536, 1u << 20,
                                 (1u << 20) + 1, 0x7fffffffu, 0x80000000u};
    for (uint32_t d : divisors) {
        const tc::FastDiv f = tc::make_fastdiv(d);
        REQUIRE(uint64_t(f.mul) == ((uint64_t(1) << f.shift) + d - 1) / d);
        const uint32_t edge[] = {0, 1, d - 1, d, d + 1, 2 * d - 1, 2 * d, 0x7ffffffeu, 0x7fffffffu};
        for (uint32_t n : edge)
            if (n < 0x80000000u) REQUIRE(tc::fastdiv(n, f) == n / d);
        for (int i = 0; i < 20000; ++i) {
            const uint32_t n = rng() & 0x7fffffffu;
            REQUIRE(tc::fastdiv(n, f) == n / d);
        }
        for (uint32_t m = 0; m < 3000; ++m)      // around multiples of d, where a wrong multiplier shows
            for (int32_t e = -1; e <= 1; ++e) {
                const uint64_t n = uint64_t(m) * d + uint64_t(int64_t(e));
                if (n < 0x80000000ull) REQUIRE(tc::fastdiv(uint32_t(n), f) == uint32_t(n) / d);
            }
    }
    // item -> (block, plane, tile)
    for (int rep = 0; rep < 200; ++rep) {
        const uint32_t tiles = 1 + rng() % 9, planes = 2 * (1 + rng() % 80), n = 1 + rng() % 40;
        const tc::FastDiv ft = tc::make_fastdiv(tiles), fp = tc::make_fastdiv(planes);
        uint32_t item = 0;
        for (uint32_t k = 0; k < n; ++k)
            for (uint32_t p = 0; p < planes; ++p)
                for (uint32_t t = 0; t < tiles; ++t, ++item) {
                    const tc::ItemPos at = tc::item_pos(item, ft, fp);
                    REQUIRE(at.k == k && at.p == p && at.t == t);
                }
    }
    // workgroup -> items, as the three kinds of launch walk them
    for (int rep = 0; rep < 3000; ++rep) {
        const uint32_t n_items = rng() % 5000;
        uint32_t grid = 1 + rng() % (rep % 3 ? 64 : 6000);
        const uint32_t chunks = grid >= tc::kXcds && rng() % 4 ? tc::kXcds : 1;
        std::vector<uint8_t> seen(n_items, 0);
        const uint32_t per = (n_items + chunks - 1) / chunks;
        for (uint32_t b = 0; b < grid; ++b) {
            const tc::ItemWalk w = tc::staged_walk(b, grid, n_items, chunks);
            REQUIRE(w.step >= 1 && w.end <= n_items);
            for (uint64_t item = w.first; item < w.end; item += w.step) {
                REQUIRE(item / per == b % chunks);          // stays inside the run of its XCD
                REQUIRE(seen[item]++ == 0);
            }
        }
        for (uint32_t i = 0; i < n_items; ++i) REQUIRE(seen[i] == 1);

        // host-bound walk: `width` items per stop over [first, n_items)
        const uint32_t first = n_items ? rng() % (n_items + 1) : 0, wgs = 1 + rng() % 40, width = 8;
        std::fill(seen.begin(), seen.end(), 0);
        for (uint32_t b = 0; b < wgs; ++b) {
            const tc::ItemWalk w = tc::strided_walk(b, wgs, first, n_items, width);
            REQUIRE(w.end == n_items && w.step == wgs * width);
            for (uint64_t item = w.first; item < w.end; item += w.step) {
                const uint32_t count = uint32_t(std::min<uint64_t>(width, w.end - item));
                for (uint32_t u = 0; u < count; ++u) REQUIRE(item + u >= first && seen[item + u]++ == 0);
            }
        }
        for (uint32_t i = 0; i < n_items; ++i) REQUIRE(seen[i] == (i >= first ? 1 : 0));
    }
    // the extremes a launch may reach: the last items of the largest grid, no wrap-around
    {
        const uint32_t n_items = 0x7fffffffu, grid = 0x7fffffffu;
        for (uint32_t b : {0u, 7u, 8u, grid - 9, grid - 8, grid - 1}) {
            const tc::ItemWalk w = tc::staged_walk(b, grid, n_items, tc::kXcds);
            REQUIRE(w.end <= n_items && uint64_t(w.first) + w.step > w.first);
            if (w.first < w.end) REQUIRE(uint64_t(w.first) + w.step >= w.end || w.step >= 1);
        }
    }
}

static void arena_stream(uint32_t seed)
{
    std::mt19937 rng(seed);
    const uint64_t N = 300;
    tc::HostArena ar(N);
    std::vector<std::pair<uint64_t, uint64_t>> live;   // (start, len)
    std::vector<char> map(N, 0);
    for (int step = 0; step < 20000; ++step) {
        if (rng() % 2 || live.empty()) {
            uint64_t n = 1 + rng() % 40;
            int64_t s = ar.alloc(n);
            if (s >= 0) {
                REQUIRE(uint64_t(s) + n <= N);
                for (uint64_t i = 0; i < n; ++i) { REQUIRE(!map[s + i]); map[s + i] = 1; }
                live.push_back({uint64_t(s), n});
                uint64_t st = 0, room = 0;
                REQUIRE(ar.locate(uint64_t(s) + n - 1, &st, &room) && st == uint64_t(s) && room == 1);
            }
        } else {
            size_t k = rng() % live.size();
            auto [s, n] = live[k];
            live.erase(live.begin() + long(k));
            const bool busy = rng() % 3 == 0;
            if (busy) ar.begin_transfer(s);
            REQUIRE(ar.free(s) == TC_OK && ar.free(s) == TC_ERR_INVAL);
            if (busy) ar.end_transfer(s);
            for (uint64_t i = 0; i < n; ++i) map[s + i] = 0;
        }
        uint64_t used = 0;
        for (char c : map) used += c;
        REQUIRE(ar.used() == used);
    }
}

static void index_threads()
{
    tc_index *ix = nullptr;
    REQUIRE(tc_index_create(&ix) == TC_OK);
    static char records[4][64 * 256];
    std::vector<std::thread> ts;
    for (int t = 0; t < 4; ++t)
        ts.emplace_back([ix, t] {
            std::mt19937 rng(100 + t);
            uint64_t keys[64];
            int32_t blocks[64];
            for (int i = 0; i < 64; ++i) { keys[i] = (uint64_t(t) << 32) | uint64_t(i); blocks[i] = i; }
            for (int round = 0; round < 400; ++round) {
                uint32_t n = 1 + rng() % 64;
                REQUIRE(tc_index_insert(ix, keys, blocks, records[t], 256, n) == TC_OK);
                REQUIRE(tc_index_insert(ix, keys, blocks, records[t], 256, 1) == TC_ERR_DUP);
                tc_index_hit hits[64];
                uint32_t h = 0;
                REQUIRE(tc_index_lookup(ix, keys, 64, hits, &h) == TC_OK && h == n);
                REQUIRE(hits[n - 1].cpu_record == records[t] + 256 * (n - 1) && hits[n - 1].state == TC_RES_CPU);
                uint64_t other[2] = {(uint64_t((t + 1) % 4) << 32), 12345};
                (void)tc_index_lookup(ix, other, 2, hits, &h);          // races with the neighbour's updates by design
                REQUIRE(tc_index_begin_upload(ix, keys, blocks, n) == TC_OK);
                REQUIRE(tc_index_pending(ix, keys, 64) == n);
                REQUIRE(tc_index_remove(ix, keys, 1) == TC_ERR_INVAL);
                REQUIRE(tc_index_finish_upload(ix, keys, n) == TC_OK);
                REQUIRE(tc_index_pending(ix, keys, 64) == 0);
            }
        });
    for (auto &t : ts) t.join();
    REQUIRE(tc_index_size(ix) == 0);
    REQUIRE(tc_index_destroy(ix) == TC_OK);
}

static void forecaster_threads()
{
    tc_forecaster *f = nullptr;
    REQUIRE(tc_forecaster_create(0.5, 0.25, 1000.0, &f) == TC_OK);
    std::vector<std::thread> ts;
    for (int t = 0; t < 4; ++t)
        ts.emplace_back([f, t] {
            for (int i = 0; i < 5000; ++i) {
                REQUIRE(tc_forecaster_observe(f, uint32_t((t + i) % 7), 10.0 + i % 50) == TC_OK);
                double e = tc_forecaster_estimate(f, uint32_t(i % 9), i % 2, 100.0);
                REQUIRE(e > 0 && e <= 1000.0);
            }
        });
    for (auto &t : ts) t.join();
    REQUIRE(tc_forecaster_destroy(f) == TC_OK);
}

static void policy_fuzz()
{
    std::mt19937 gen(7);
    auto rng = [&gen]() { return uint32_t(gen()); };
    tc_cost_model m{0.05, 0.0374, 0.07, 0.0375};
    for (int i = 0; i < 20000; ++i) {
        tc_waiting_req q[6];
        uint32_t nq = rng() % 7;
        for (uint32_t k = 0; k < nq && k < 6; ++k) q[k] = tc_waiting_req{rng() % 600u, double(rng() % 50000u)};
        if (nq > 6) nq = 6;
        tc_gate_input in{rng() % 600, rng() % 800, rng() % 1000, 1 + rng() % 1000, (rng() % 11) / 10.0, double(rng() % 3000), 0.1 + (rng() % 400) / 10.0};
        int32_t chosen = -2;
        int reason = -1;
        int rc = tc_offload_gate(&m, &in, q, nq, &chosen, &reason);
        REQUIRE((rc == 1 && reason == TC_GATE_PASS && chosen >= 0 && uint32_t(chosen) < nq) || (rc == 0 && reason >= 1 && reason <= 4 && chosen == -1));
        tc_upload_cand c[9];
        uint32_t n = rng() % 10, order[9], reserve[9];
        if (n > 9) n = 9;
        for (uint32_t k = 0; k < n; ++k) c[k] = tc_upload_cand{(rng() % 5) / 4.0, (rng() % 5) / 4.0, rng() % 3000};
        uint32_t gf = rng() % 4000, dc = rng() % 4000, sf = rng() % 4000;
        REQUIRE(tc_upload_plan(c, n, gf, dc, sf, order, reserve) == TC_OK);
        uint64_t sum = 0;
        std::set<uint32_t> seen;
        for (uint32_t k = 0; k < n; ++k) { sum += reserve[k]; seen.insert(order[k]); REQUIRE(order[k] < n); }
        REQUIRE(seen.size() == n && sum <= tc_upload_budget(gf, dc, sf));
    }
    int32_t toks[100];
    for (int i = 0; i < 100; ++i) toks[i] = i * 31;
    uint64_t keys[6], nk = 0;
    REQUIRE(tc_chain_hashes(toks, 100, 16, 0, keys, &nk) == TC_OK && nk == 6);
    tc_req_state r{TC_RUNNING, 0, 0, 0};
    int act = 0;
    for (int i = 0; i < 100000; ++i) (void)tc_lifecycle_step(&r, int(rng() % 8), &act);
    REQUIRE(r.state <= TC_UPLOADED);
}

int main()
{
    for (uint32_t s = 1; s <= 3; ++s) { block_pool_stream(s); arena_stream(s); }
    item_mapping(11);
    index_threads();
    forecaster_threads();
    policy_fuzz();
    std::puts("ok");
    return 0;
}
