// Concurrency check of the pool's host side: the header promises that a pool may be used from
// several threads at once (one lock per pool).  Eight threads allocate, free, range-check, read
// the bounds table and attach / detach tenants on one pool; the program is built with the
// thread sanitizer, and again with the address and undefined-behaviour sanitizers, by tests/test_boundary_host.py, and it checks on its own that allocations
// of one tenant never overlap, stay inside the partition, and coalesce back into one block.
// Exit status 0 = all invariants held (a sanitizer report ends the run with its own status).
#include <atomic>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <thread>
#include <utility>
#include <vector>

#include "../../paper_2401_09290_amd/csrc/pool.hpp"

static std::atomic<int> failures{0};
#define EXPECT(cond)                                                          \
    do {                                                                      \
        if (!(cond)) {                                                        \
            std::fprintf(stderr, "line %d: %s\n", __LINE__, #cond);           \
            failures.fetch_add(1);                                            \
        }                                                                     \
    } while (0)

static uint64_t next(uint64_t &s) { s = s * 6364136223846793005ull + 1442695040888963407ull; return s >> 33; }

int main()
{
    const uint64_t MiB = 1ull << 20, base = 1ull << 40;
    const uint64_t sizes[2] = {16 * MiB, 16 * MiB};
    gd::Pool *pool = nullptr;
    if (gd::pool_create(base, 64 * MiB, sizes, 2, false, &pool) != GD_OK) return 2;
    const int THREADS = 8, ROUNDS = 4000;
    // tenants 0 and 1 are shared by four threads each; every thread also attaches and detaches tenants of its own
    std::vector<std::vector<std::pair<uint64_t, uint64_t>>> kept(THREADS);
    std::vector<std::thread> pool_threads;
    for (int t = 0; t < THREADS; ++t)
        pool_threads.emplace_back([&, t]() {
            uint64_t seed = 1234 + t;
            const int tenant = t & 1;
            std::vector<std::pair<uint64_t, uint64_t>> mine;
            uint64_t pb, ps, pm;
            for (int r = 0; r < ROUNDS; ++r) {
                const uint64_t what = next(seed) % 8;
                if (what < 4 || mine.empty()) {
                    const uint64_t bytes = 256 * (1 + next(seed) % 64), align = 256ull << (next(seed) % 4);
                    uint64_t p = 0;
                    const int rc = gd::alloc(pool, tenant, bytes, align, &p);
                    EXPECT(rc == GD_OK || rc == GD_ENOMEM);
                    if (rc == GD_OK) {
                        EXPECT(p % align == 0 && gd::check_copy(pool, tenant, p, bytes) == GD_OK);
                        EXPECT(gd::check_copy(pool, 1 - tenant, p, bytes) == GD_ERANGE);
                        mine.emplace_back(p, bytes);
                    }
                } else if (what < 7) {
                    const size_t k = next(seed) % mine.size();
                    EXPECT(gd::free_(pool, tenant, mine[k].first) == GD_OK);
                    mine[k] = mine.back();
                    mine.pop_back();
                } else {
                    // a tenant of this thread's own comes and goes; the shared tenants' rows must not move
                    int own = -1;
                    const int rc = gd::tenant_attach(pool, MiB, &own);
                    EXPECT(rc == GD_OK || rc == GD_ENOMEM);
                    if (rc == GD_OK) {
                        uint64_t q = 0;
                        EXPECT(own >= 2 && gd::alloc(pool, own, 4096, 256, &q) == GD_OK);
                        EXPECT(gd::tenant_detach(pool, own) == GD_EBUSY);
                        EXPECT(gd::free_(pool, own, q) == GD_OK);
                        EXPECT(gd::free_(pool, own, q) == GD_EINVAL);                 // second free of the same block
                        EXPECT(gd::tenant_detach(pool, own) == GD_OK);
                    }
                }
                EXPECT(gd::partition_info(pool, tenant, &pb, &ps, &pm) == GD_OK && pb == base + tenant * 16 * MiB && ps == 16 * MiB);
                gd::LaunchRow row;
                EXPECT(gd::launch_row(pool, tenant, &row) == GD_OK && row.base == pb && row.size == ps);
            }
            kept[t] = mine;
        });
    for (auto &th : pool_threads) th.join();
    // what the threads still hold: inside the partition and pairwise disjoint per tenant
    for (int tenant = 0; tenant < 2; ++tenant) {
        std::vector<std::pair<uint64_t, uint64_t>> all;
        for (int t = tenant; t < THREADS; t += 2) all.insert(all.end(), kept[t].begin(), kept[t].end());
        const uint64_t pb = base + tenant * 16 * MiB;
        for (size_t i = 0; i < all.size(); ++i) {
            EXPECT(all[i].first >= pb && all[i].first + all[i].second <= pb + 16 * MiB);
            for (size_t j = i + 1; j < all.size(); ++j)
                EXPECT(all[i].first + all[i].second <= all[j].first || all[j].first + all[j].second <= all[i].first);
        }
        for (auto &b : all) EXPECT(gd::free_(pool, tenant, b.first) == GD_OK);
        uint64_t whole = 0;                                   // everything coalesced: the whole partition is one block again
        EXPECT(gd::alloc(pool, tenant, 16 * MiB, 256, &whole) == GD_OK && whole == pb);
    }
    delete pool;                                              // what gd_pool_destroy does
    std::printf("threads %d rounds %d failures %d\n", THREADS, ROUNDS, failures.load());
    return failures.load() ? 1 : 0;
}
