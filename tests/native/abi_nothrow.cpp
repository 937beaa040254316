// Allocation-failure check of the C ABI: the header promises that nothing throws or aborts across it
// and that host allocation failure is reported as GD_ENOMEM with out-parameters untouched.  This
// program replaces the global operator new (the library's allocations resolve to it) with one that
// fails on the k-th allocation after arming, and calls each entry point that allocates with k = 0, 1,
// 2, ... until the call succeeds.  Every failing call must return GD_ENOMEM and leave the pool usable.
// Built and run by tests/test_boundary_host.py; needs no GPU (no kernel is launched).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <new>

#include "../../include/guardian.h"

static long countdown = -1;          // < 0: not armed
static long failures_injected = 0;

void *operator new(std::size_t n)
{
    if (countdown == 0) {
        countdown = -1;
        ++failures_injected;
        throw std::bad_alloc();
    }
    if (countdown > 0) --countdown;
    if (void *p = std::malloc(n ? n : 1)) return p;
    throw std::bad_alloc();
}
void *operator new(std::size_t n, const std::nothrow_t &) noexcept
{
    if (countdown == 0) {
        countdown = -1;
        ++failures_injected;
        return nullptr;
    }
    if (countdown > 0) --countdown;
    return std::malloc(n ? n : 1);
}
void operator delete(void *p) noexcept { std::free(p); }
void operator delete(void *p, std::size_t) noexcept { std::free(p); }

static int bad = 0;
#define EXPECT(cond)                                                   \
    do {                                                               \
        if (!(cond)) {                                                 \
            std::fprintf(stderr, "line %d: %s\n", __LINE__, #cond);    \
            ++bad;                                                     \
        }                                                              \
    } while (0)

// Calls `call` with the k-th allocation failing, k = 0, 1, ..., until it returns GD_OK; returns how many k failed.
template <typename F, typename G>
static int until_ok(F call, G untouched)
{
    for (int k = 0; k < 64; ++k) {
        countdown = k;
        const int rc = call();
        countdown = -1;
        if (rc == GD_OK) return k;
        EXPECT(rc == GD_ENOMEM);
        EXPECT(untouched());
    }
    EXPECT(!"no success within 64 allocations");
    return -1;
}

int main()
{
    const uint64_t MiB = 1ull << 20, base = 1ull << 40;
    const uint64_t sizes[3] = {4 * MiB, 2 * MiB, 2 * MiB};
    gd_pool *pool = nullptr;
    const int k_create = until_ok([&] { return gd_pool_create(base, 16 * MiB, sizes, 3, &pool); }, [&] { return pool == nullptr; });
    EXPECT(pool != nullptr && k_create > 0);
    uint64_t p = 0;
    const int k_alloc = until_ok([&] { return gd_alloc(pool, 1, 4096, 256, &p); }, [&] { return p == 0; });
    EXPECT(p != 0 && k_alloc > 0);
    // a second block, then free the first: the free list gains a node (an allocation that may fail)
    uint64_t q = 0;
    EXPECT(gd_alloc(pool, 1, 8192, 256, &q) == GD_OK);
    const int k_free = until_ok([&] { return gd_free(pool, 1, p); }, [&] { return gd_check_copy(pool, 1, p, 4096) == GD_OK; });
    EXPECT(k_free >= 0);
    EXPECT(gd_free(pool, 1, p) == GD_EINVAL);                 // freed exactly once, whatever failed on the way
    // an aligned allocation from the middle of a free block leaves a remainder on both sides: two nodes to allocate,
    // and a failure on the second must take the first back
    uint64_t small = 0, mid = 0;
    EXPECT(gd_alloc(pool, 2, 256, 256, &small) == GD_OK);
    const int k_mid = until_ok([&] { return gd_alloc(pool, 2, 4096, 65536, &mid); }, [&] { return mid == 0; });
    EXPECT(k_mid == 2 && mid % 65536 == 0 && mid > small);
    EXPECT(gd_free(pool, 2, mid) == GD_OK && gd_free(pool, 2, small) == GD_OK);
    uint64_t all2 = 0;
    EXPECT(gd_alloc(pool, 2, 2 * MiB, 256, &all2) == GD_OK && gd_free(pool, 2, all2) == GD_OK);   // nothing was lost on the way
    int tenant = -1;
    const int k_attach = until_ok([&] { return gd_tenant_attach(pool, 2 * MiB, &tenant); }, [&] { return tenant == -1; });
    EXPECT(tenant == 3 && k_attach >= 0);
    // the pool is intact after all of that: rows where they were, the heap consistent
    uint64_t b = 0, s = 0, m = 0;
    EXPECT(gd_partition_info(pool, 0, &b, &s, &m) == GD_OK && b == base && s == 4 * MiB && m == 4 * MiB - 1);
    EXPECT(gd_free(pool, 1, q) == GD_OK);
    uint64_t whole = 0;
    EXPECT(gd_alloc(pool, 1, 2 * MiB, 256, &whole) == GD_OK);
    EXPECT(gd_tenant_detach(pool, 3) == GD_OK);
    EXPECT(gd_pool_destroy(pool) == GD_OK);
    std::printf("injected %ld allocation failures (create %d, alloc %d, split alloc %d, free %d, attach %d), problems %d\n",
                failures_injected, k_create, k_alloc, k_mid, k_free, k_attach, bad);
    return bad ? 1 : 0;
}
