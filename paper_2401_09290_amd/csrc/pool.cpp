// Host side of libguardian: partition bounds table, in-partition allocator,
// transfer range check, host twin of the fence.  Pure C++17, no HIP calls: the
// pool's device memory is never touched from here.
#include "pool.hpp"

#include <algorithm>
#include <memory>
#include <new>

namespace gd {

static inline bool is_pow2(uint64_t v) { return v && !(v & (v - 1)); }

// Smallest multiple of `align` (a power of two) that is >= v; false on overflow.
static inline bool align_up(uint64_t v, uint64_t align, uint64_t *out)
{
    uint64_t r = (v + (align - 1)) & ~(align - 1);
    if (r < v) return false;
    *out = r;
    return true;
}

static inline bool size_ok(const Pool &p, uint64_t bytes)
{
    if (bytes < GD_MIN_PARTITION) return false;
    return p.flex ? (bytes % GD_GRANULE) == 0 : is_pow2(bytes);
}

// Lowest aligned address whose block fits the pool and overlaps no attached
// partition; aligned to the size (power-of-two pools) or to the granule (flex
// pools).  `rows` need not be sorted.
static bool place(const Pool &p, uint64_t size, uint64_t *where)
{
    const uint64_t align = p.flex ? (uint64_t)GD_GRANULE : size;
    std::vector<std::pair<uint64_t, uint64_t>> taken;   // (base, end) sorted by base
    for (const Partition &r : p.rows)
        if (r.attached) taken.emplace_back(r.base, r.base + r.size);
    std::sort(taken.begin(), taken.end());

    const uint64_t pool_end = p.dev_base + p.dev_bytes;   // caller checked: no overflow
    uint64_t a;
    if (!align_up(p.dev_base, align, &a)) return false;
    size_t k = 0;
    while (a <= pool_end && pool_end - a >= size) {
        while (k < taken.size() && taken[k].second <= a) ++k;      // entirely in front of a
        if (k == taken.size() || taken[k].first >= a + size) {
            *where = a;
            return true;
        }
        if (!align_up(taken[k].second, align, &a)) return false;   // hop behind the obstacle
    }
    return false;
}

int pool_create(uint64_t dev_base, uint64_t dev_bytes, const uint64_t *part_bytes, int n, bool flex,
                Pool **out)
{
    if (!out || n < 0 || (n > 0 && !part_bytes)) return GD_EINVAL;
    if (dev_base + dev_bytes < dev_base) return GD_EINVAL;           // range wraps 2^64

    std::unique_ptr<Pool> p(new (std::nothrow) Pool);      // freed on every early return and if anything below throws
    if (!p) return GD_ENOMEM;
    p->dev_base = dev_base;
    p->dev_bytes = dev_bytes;
    p->flex = flex;
    for (int i = 0; i < n; ++i)
        if (!size_ok(*p, part_bytes[i])) return GD_ENOTPOW2;
    p->rows.resize(n);

    // power-of-two pools: by decreasing size (packs without gaps); flex pools: tenant order
    std::vector<int> order(n);
    for (int i = 0; i < n; ++i) order[i] = i;
    if (!flex)
        std::stable_sort(order.begin(), order.end(),
                         [&](int x, int y) { return part_bytes[x] > part_bytes[y]; });
    for (int t : order) {
        uint64_t where;
        if (!place(*p, part_bytes[t], &where)) return GD_ENOMEM;
        Partition &r = p->rows[t];
        r.attached = true;
        r.base = where;
        r.size = part_bytes[t];
        r.free_blocks.clear();
        r.free_blocks[where] = part_bytes[t];
        r.live.clear();
    }
    *out = p.release();
    return GD_OK;
}

int tenant_attach(Pool *p, uint64_t bytes, int *tenant_out)
{
    if (!p || !tenant_out) return GD_EINVAL;
    if (!size_ok(*p, bytes)) return GD_ENOTPOW2;
    std::lock_guard<std::mutex> g(p->mu);
    uint64_t where;
    if (!place(*p, bytes, &where)) return GD_ENOMEM;
    size_t slot = 0;
    while (slot < p->rows.size() && p->rows[slot].attached) ++slot;
    // what can fail (host allocations) comes first and changes nothing; the row is then filled in without allocating
    std::map<uint64_t, uint64_t> whole;
    whole.emplace(where, bytes);
    if (slot == p->rows.size()) p->rows.emplace_back();
    Partition &r = p->rows[slot];
    r.attached = true;
    r.base = where;
    r.size = bytes;
    r.free_blocks.swap(whole);
    r.live.clear();
    *tenant_out = (int)slot;
    return GD_OK;
}

int set_fault_counters(Pool *p, uint64_t dev_counters, int slots)
{
    if (!p || slots < 0 || (dev_counters & 7)) return GD_EINVAL;
    const uint64_t bytes = 8 * (uint64_t)slots;
    if (dev_counters + bytes < dev_counters) return GD_EINVAL;
    // must not overlap the pool: no tenant may be able to address its own counter
    if (slots > 0 && dev_counters < p->dev_base + p->dev_bytes && p->dev_base < dev_counters + bytes) return GD_EINVAL;
    std::lock_guard<std::mutex> g(p->mu);
    p->fault_counters = slots ? dev_counters : 0;
    p->fault_slots = slots;
    return GD_OK;
}

static Partition *row_of(Pool *p, int tenant)
{
    if (tenant < 0 || (size_t)tenant >= p->rows.size() || !p->rows[tenant].attached) return nullptr;
    return &p->rows[tenant];
}

int tenant_detach(Pool *p, int tenant)
{
    if (!p) return GD_EINVAL;
    std::lock_guard<std::mutex> g(p->mu);
    Partition *r = row_of(p, tenant);
    if (!r) return GD_ENOTENANT;
    if (!r->live.empty()) return GD_EBUSY;
    r->attached = false;
    r->free_blocks.clear();
    return GD_OK;
}

int partition_info(const Pool *p, int tenant, uint64_t *base, uint64_t *size, uint64_t *mask)
{
    if (!p) return GD_EINVAL;
    std::lock_guard<std::mutex> g(p->mu);
    const Partition *r = row_of(const_cast<Pool *>(p), tenant);
    if (!r) return GD_ENOTENANT;
    if (base) *base = r->base;
    if (size) *size = r->size;
    if (mask) *mask = r->size - 1;
    return GD_OK;
}

int launch_row(const Pool *p, int tenant, LaunchRow *out)
{
    if (!p || !out) return GD_EINVAL;
    std::lock_guard<std::mutex> g(p->mu);
    const Partition *r = row_of(const_cast<Pool *>(p), tenant);
    if (!r) return GD_ENOTENANT;
    *out = LaunchRow{r->base, r->size, p->flex, p->fault_counters, p->fault_slots};
    return GD_OK;
}

int alloc(Pool *p, int tenant, uint64_t bytes, uint64_t align, uint64_t *dptr_out)
{
    if (!p || !dptr_out || bytes == 0 || !is_pow2(align)) return GD_EINVAL;
    if (align < GD_GRANULE) align = GD_GRANULE;
    uint64_t need;
    if (!align_up(bytes, GD_GRANULE, &need)) return GD_ENOMEM;
    std::lock_guard<std::mutex> g(p->mu);
    Partition *r = row_of(p, tenant);
    if (!r) return GD_ENOTENANT;
    for (auto it = r->free_blocks.begin(); it != r->free_blocks.end(); ++it) {
        const uint64_t start = it->first, len = it->second, stop = start + len;
        uint64_t at;
        if (!align_up(start, align, &at) || at >= stop || stop - at < need) continue;
        // split: [start, at) stays free, [at, at+need) is taken, [at+need, stop) stays free.  The steps that
        // allocate a node come first and are undone if a later one fails; the rest cannot fail.
        auto taken = r->live.emplace(at, need).first;
        if (at > start && at + need < stop) {              // two remainders: one new node
            try {
                r->free_blocks.emplace(at + need, stop - (at + need));
            } catch (...) {
                r->live.erase(taken);
                throw;
            }
            it->second = at - start;
        } else if (at > start) {                           // front remainder only: the node shrinks
            it->second = at - start;
        } else if (at + need < stop) {                     // back remainder only: the node moves
            auto node = r->free_blocks.extract(it);
            node.key() = at + need;
            node.mapped() = stop - (at + need);
            r->free_blocks.insert(std::move(node));
        } else {
            r->free_blocks.erase(it);
        }
        *dptr_out = at;
        return GD_OK;
    }
    return GD_ENOMEM;
}

int free_(Pool *p, int tenant, uint64_t dptr)
{
    if (!p) return GD_EINVAL;
    std::lock_guard<std::mutex> g(p->mu);
    Partition *r = row_of(p, tenant);
    if (!r) return GD_ENOTENANT;
    auto it = r->live.find(dptr);
    if (it == r->live.end()) return GD_EINVAL;
    uint64_t start = it->first, len = it->second;
    auto node = r->live.extract(it);          // kept: it becomes the free list's node if no neighbour absorbs the block (no allocation, cannot fail)
    // merge with the free block behind and the one in front
    auto next = r->free_blocks.lower_bound(start);
    if (next != r->free_blocks.end() && next->first == start + len) {
        len += next->second;
        next = r->free_blocks.erase(next);
    }
    if (next != r->free_blocks.begin()) {
        auto prev = std::prev(next);
        if (prev->first + prev->second == start) {
            prev->second += len;
            return GD_OK;
        }
    }
    node.mapped() = len;
    r->free_blocks.insert(std::move(node));
    return GD_OK;
}

int check_copy(const Pool *p, int tenant, uint64_t dptr, uint64_t bytes)
{
    if (!p) return GD_EINVAL;
    std::lock_guard<std::mutex> g(p->mu);
    const Partition *r = row_of(const_cast<Pool *>(p), tenant);
    if (!r) return GD_ENOTENANT;
    if (dptr < r->base) return GD_ERANGE;
    if (bytes > r->size) return GD_ERANGE;
    if (dptr - r->base > r->size - bytes) return GD_ERANGE;
    return GD_OK;
}

uint64_t fence_host(uint64_t base, uint64_t size, uint64_t addr, uint32_t width, int mode)
{
    const uint64_t bad = ~uint64_t(0);
    if (!(width == 1 || width == 2 || width == 4 || width == 8 || width == 16) || size == 0) return bad;
    switch (mode) {
    case GD_FENCE_NONE:
        return addr;
    case GD_FENCE_BITWISE:
        if (!is_pow2(size) || (base & (size - 1))) return bad;
        return (addr & (size - 1) & ~uint64_t(width - 1)) | base;
    case GD_FENCE_MODULO:
        return base + (((addr - base) % size) & ~uint64_t(width - 1));
    case GD_FENCE_CHECK: {
        const uint64_t last = addr + (width - 1);
        if (addr < base || last < addr || last > base + (size - 1)) return bad;
        return addr;
    }
    case GD_FENCE_HWCHECK: {
        if (size > 0xffffffffull) return bad;
        const uint64_t off = ((addr - base) & 0xffffffffull) & ~uint64_t(width - 1);
        return off + width <= size ? base + off : bad;
    }
    default:
        return bad;
    }
}

}  // namespace gd
