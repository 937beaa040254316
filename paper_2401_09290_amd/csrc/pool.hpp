// Host-side state of a pool: the partition bounds table (paper Section 4.2.1)
// and, per partition, a free list and the live allocations.  Host memory only.
#pragma once

#include <cstdint>
#include <map>
#include <mutex>
#include <vector>

#include "../../include/guardian.h"

namespace gd {

struct Partition {
    bool attached = false;
    uint64_t base = 0;
    uint64_t size = 0;                       // power of two, base % size == 0
    std::map<uint64_t, uint64_t> free_blocks;  // start -> bytes, address ordered, never adjacent
    std::map<uint64_t, uint64_t> live;         // start -> bytes (rounded to the granule)
};

}  // namespace gd

// The opaque handle of the C ABI.
struct gd_pool {
    uint64_t dev_base = 0;
    uint64_t dev_bytes = 0;
    std::vector<gd::Partition> rows;         // index = tenant number
    bool flex = false;                       // arbitrary sizes (modulo fence / checking only)
    uint64_t fault_counters = 0;             // device address of the per-tenant uint64 counters, 0 = none
    int fault_slots = 0;
    mutable std::mutex mu;
};

namespace gd {

using Pool = ::gd_pool;

int pool_create(uint64_t dev_base, uint64_t dev_bytes, const uint64_t *part_bytes, int n, bool flex, Pool **out);
int set_fault_counters(Pool *p, uint64_t dev_counters, int slots);
int tenant_attach(Pool *p, uint64_t bytes, int *tenant_out);
int tenant_detach(Pool *p, int tenant);
int partition_info(const Pool *p, int tenant, uint64_t *base, uint64_t *size, uint64_t *mask);

// Everything a launch needs from the pool, read in one go under the pool's lock.
struct LaunchRow {
    uint64_t base, size;
    bool flex;
    uint64_t fault_counters;
    int fault_slots;
};
int launch_row(const Pool *p, int tenant, LaunchRow *out);
int alloc(Pool *p, int tenant, uint64_t bytes, uint64_t align, uint64_t *dptr_out);
int free_(Pool *p, int tenant, uint64_t dptr);
int check_copy(const Pool *p, int tenant, uint64_t dptr, uint64_t bytes);
uint64_t fence_host(uint64_t base, uint64_t size, uint64_t addr, uint32_t width, int mode);

}  // namespace gd
