// extern "C" surface of libguardian (see include/guardian.h) and the kernel
// registry: kernel id -> {name, size of its argument block, launcher}.  The
// registry plays the role of the paper's pointerToSymbol map (Section 4.2.3):
// at launch the manager looks the sandboxed kernel up, extends the parameters
// by the tenant's base and mask taken from the partition bounds table, and
// issues it on the tenant's stream; a tenant that runs with protection off
// gets the native (unfenced) build of the same kernel.
#include <hip/hip_runtime.h>

#include <chrono>
#include <cstring>
#include <new>

#include "launchers.hpp"
#include "pool.hpp"

namespace gd {

static thread_local int g_last_hip_error = 0;
void note_hip_error(hipError_t e) { g_last_hip_error = (int)e; }

struct KernelEntry {
    const char *name;
    size_t args_bytes;
    Launcher launch;
};

static const KernelEntry g_registry[GD_K_COUNT] = {
    /* GD_K_STORE_TID       */ {"store_tid", sizeof(gd_args_store_tid), launch_store_tid},
    /* GD_K_FENCE_ADDRS     */ {"fence_addrs", sizeof(gd_args_fence_addrs), launch_fence_addrs},
    /* GD_K_COPY            */ {"copy", sizeof(gd_args_copy), launch_copy},
    /* GD_K_TRIAD           */ {"triad", sizeof(gd_args_triad), launch_triad},
    /* GD_K_SAXPY_IDX       */ {"saxpy_idx", sizeof(gd_args_saxpy_idx), launch_saxpy_idx},
    /* GD_K_GATHER32_I64    */ {"gather32_i64", sizeof(gd_args_gather), launch_gather32_i64},
    /* GD_K_SCATTER_F32_I64 */ {"scatter_f32_i64", sizeof(gd_args_scatter), launch_scatter_f32_i64},
    /* GD_K_GATHER32_I32    */ {"gather32_i32", sizeof(gd_args_gather), launch_gather32_i32},
    /* GD_K_SUM_F32         */ {"sum_f32", sizeof(gd_args_sum), launch_sum_f32},
    /* GD_K_RMSNORM_BF16    */ {"rmsnorm_bf16", sizeof(gd_args_rmsnorm), launch_rmsnorm_bf16},
    /* GD_K_GEMM_BF16       */ {"gemm_bf16", sizeof(gd_args_gemm), launch_gemm_bf16},
    /* GD_K_CHASE           */ {"chase", sizeof(gd_args_chase), launch_chase},
};

}  // namespace gd

// Nothing may leave an extern "C" function by exception: the host containers
// (std::vector, std::map) can throw std::bad_alloc, which is reported as GD_ENOMEM.
#define GD_ABI_GUARD(expr)                                  \
    try {                                                   \
        return (expr);                                      \
    } catch (const std::bad_alloc &) {                      \
        return GD_ENOMEM;                                   \
    } catch (...) {                                         \
        return GD_EINVAL;                                   \
    }

static int create_pool(uint64_t dev_base, uint64_t dev_bytes, const uint64_t *part_bytes, int n_tenants,
                       bool flex, gd_pool **out)
{
    if (!out) return GD_EINVAL;
    gd::Pool *p = nullptr;
    const int rc = gd::pool_create(dev_base, dev_bytes, part_bytes, n_tenants, flex, &p);
    if (rc == GD_OK) *out = p;
    return rc;
}

extern "C" {

int gd_pool_create(uint64_t dev_base, uint64_t dev_bytes, const uint64_t *part_bytes, int n_tenants,
                   gd_pool **out)
{
    GD_ABI_GUARD(create_pool(dev_base, dev_bytes, part_bytes, n_tenants, false, out))
}

int gd_pool_create_flex(uint64_t dev_base, uint64_t dev_bytes, const uint64_t *part_bytes, int n_tenants,
                        gd_pool **out)
{
    GD_ABI_GUARD(create_pool(dev_base, dev_bytes, part_bytes, n_tenants, true, out))
}

int gd_pool_set_fault_counters(gd_pool *pool, uint64_t dev_counters, int slots)
{
    GD_ABI_GUARD(gd::set_fault_counters(pool, dev_counters, slots))
}

int gd_pool_destroy(gd_pool *pool)
{
    if (!pool) return GD_EINVAL;
    delete pool;
    return GD_OK;
}

int gd_tenant_attach(gd_pool *pool, uint64_t bytes, int *tenant_out) { GD_ABI_GUARD(gd::tenant_attach(pool, bytes, tenant_out)) }
int gd_tenant_detach(gd_pool *pool, int tenant) { GD_ABI_GUARD(gd::tenant_detach(pool, tenant)) }

int gd_partition_info(const gd_pool *pool, int tenant, uint64_t *base, uint64_t *size, uint64_t *mask)
{
    GD_ABI_GUARD(gd::partition_info(pool, tenant, base, size, mask))
}

int gd_alloc(gd_pool *pool, int tenant, uint64_t bytes, uint64_t align, uint64_t *dptr_out)
{
    GD_ABI_GUARD(gd::alloc(pool, tenant, bytes, align, dptr_out))
}

int gd_free(gd_pool *pool, int tenant, uint64_t dptr) { GD_ABI_GUARD(gd::free_(pool, tenant, dptr)) }

int gd_check_copy(const gd_pool *pool, int tenant, uint64_t dptr, uint64_t bytes)
{
    GD_ABI_GUARD(gd::check_copy(pool, tenant, dptr, bytes))
}

uint64_t gd_fence_host(uint64_t base, uint64_t size, uint64_t addr, uint32_t width, int mode)
{
    return gd::fence_host(base, size, addr, width, mode);
}

int gd_kernel_count(void) { return GD_K_COUNT; }

const char *gd_kernel_name(int id) { return (id >= 0 && id < GD_K_COUNT) ? gd::g_registry[id].name : nullptr; }

size_t gd_kernel_args_bytes(int id) { return (id >= 0 && id < GD_K_COUNT) ? gd::g_registry[id].args_bytes : 0; }

// Bounds table row of the launching tenant -> the extra kernel parameters and the
// kernel variant for `mode` (the parameter augmentation of Section 4.2.3).
static int fence_args_for(gd_pool *pool, int tenant, int mode, int *variant, gd::FenceArgs *extra)
{
    gd::LaunchRow row;
    const int rc = gd::launch_row(pool, tenant, &row);                       // under the pool's lock
    if (rc != GD_OK) return rc;
    const uint64_t base = row.base, size = row.size, mask = row.size - 1;
    *extra = gd::FenceArgs{base, mask, 0, 0, (uint32_t)tenant, 0};
    switch (mode) {
    case GD_FENCE_NONE:
        *variant = gd::V_NONE;
        return GD_OK;
    case GD_FENCE_BITWISE:
        if (row.flex) return GD_EINVAL;              // needs power-of-two, size-aligned partitions
        // A mask that fits 32 bits lets the kernel fence a 32-bit offset and add
        // the base in the addressing mode; larger partitions fence the high word.
        *variant = (mask <= 0xffffffffull) ? gd::V_BIT32 : gd::V_BIT64;
        return GD_OK;
    case GD_FENCE_MODULO: {
        // Reciprocal for the exact 64-bit remainder by `size` (division by an
        // invariant integer, round-up method): shift = ceil(log2 size),
        // magic = floor(2^64 * (2^shift - size) / size) + 1.
        *variant = gd::V_MOD;
        uint32_t l = 0;
        while (l < 64 && ((uint64_t)1 << l) < size) ++l;
        const unsigned __int128 pow_l = (unsigned __int128)1 << l;
        extra->mask = size;
        extra->shift = l;
        extra->magic = (uint64_t)((((unsigned __int128)1 << 64) * (pow_l - size)) / size) + 1;
        return GD_OK;
    }
    case GD_FENCE_CHECK:
        if (!row.fault_counters || tenant >= row.fault_slots) return GD_EINVAL;
        *variant = gd::V_CHECK;
        extra->mask = size;
        extra->faults = row.fault_counters;
        return GD_OK;
    case GD_FENCE_HWCHECK:
        // the descriptor's num_records is a 32-bit byte count
        if (size > 0xffffffffull) return GD_ESHAPE;
        *variant = gd::V_BUF;
        extra->mask = size;
        return GD_OK;
    default:
        return GD_ENOKERNEL;
    }
}

static int launch_fenced(gd_pool *pool, int tenant, int kernel_id, const void *args, size_t args_bytes,
                         const uint32_t grid[3], const uint32_t block[3], void *hip_stream, int mode)
{
    if (!pool || !args) return GD_EINVAL;
    if (kernel_id < 0 || kernel_id >= GD_K_COUNT) return GD_ENOKERNEL;
    const gd::KernelEntry &k = gd::g_registry[kernel_id];                    // lookup
    if (args_bytes != k.args_bytes) return GD_EINVAL;

    int variant;
    gd::FenceArgs extra;
    const int rc = fence_args_for(pool, tenant, mode, &variant, &extra);
    if (rc != GD_OK) return rc;

    alignas(16) unsigned char copy[64];                                      // parameter augmentation
    static_assert(sizeof(gd_args_gemm) <= sizeof(copy) && sizeof(gd_args_scatter) <= sizeof(copy), "args copy too small");
    std::memcpy(copy, args, args_bytes);
    const gd::Shape shape = {grid, block};
    return k.launch(copy, extra, variant, shape, static_cast<hipStream_t>(hip_stream));
}

static int sum_noalloc(gd_pool *pool, int tenant, uint64_t out, uint64_t in, uint64_t n, void *hip_stream, int mode)
{
    if (!pool) return GD_EINVAL;
    if (n > GD_SUM_NOALLOC_MAX_N) return GD_ESHAPE;
    int variant;
    gd::FenceArgs extra;
    const int rc = fence_args_for(pool, tenant, mode, &variant, &extra);
    if (rc != GD_OK) return rc;
    return gd::launch_sum_f32_noalloc(out, in, n, extra, variant, static_cast<hipStream_t>(hip_stream));
}

static int probe_host_path(gd_pool *pool, int tenant, uint64_t dptr, uint32_t iters, void *hip_stream, int mode, double *ns)
{
    if (!pool || !ns || !dptr || iters == 0 || iters > (1u << 20)) return GD_EINVAL;
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    int variant;
    gd::FenceArgs extra;
    int rc = fence_args_for(pool, tenant, mode, &variant, &extra);
    if (rc != GD_OK) return rc;
    double out[3];
    const gd_args_store_tid none = {dptr, 0, 1, 0}, some = {dptr, 64, 1, 0};
    auto sync = [&]() {
        const hipError_t e = hipStreamSynchronize(stream);
        if (e != hipSuccess) gd::note_hip_error(e);
        return e == hipSuccess ? GD_OK : GD_EHIP;
    };
    auto timed = [&](const gd_args_store_tid &a, double *per_call) {
        if ((rc = sync()) != GD_OK) return rc;
        const auto t0 = std::chrono::steady_clock::now();
        for (uint32_t i = 0; i < iters && rc == GD_OK; ++i)
            rc = launch_fenced(pool, tenant, GD_K_STORE_TID, &a, sizeof a, nullptr, nullptr, hip_stream, mode);
        const auto t1 = std::chrono::steady_clock::now();
        *per_call = std::chrono::duration<double, std::nano>(t1 - t0).count() / iters;
        return rc;
    };
    if ((rc = timed(none, &out[0])) != GD_OK) return rc;
    if ((rc = timed(some, &out[1])) != GD_OK) return rc;
    if ((rc = sync()) != GD_OK) return rc;
    if ((rc = gd::probe_raw_launches(some, extra, variant, iters, stream, &out[2])) != GD_OK) return rc;
    if ((rc = sync()) != GD_OK) return rc;
    std::memcpy(ns, out, sizeof out);
    return GD_OK;
}

int gd_launch_fenced(gd_pool *pool, int tenant, int kernel_id, const void *args, size_t args_bytes,
                     const uint32_t grid[3], const uint32_t block[3], void *hip_stream, int mode)
{
    GD_ABI_GUARD(launch_fenced(pool, tenant, kernel_id, args, args_bytes, grid, block, hip_stream, mode))
}

int gd_sum_f32_noalloc(gd_pool *pool, int tenant, uint64_t out, uint64_t in, uint64_t n, void *hip_stream, int mode)
{
    GD_ABI_GUARD(sum_noalloc(pool, tenant, out, in, n, hip_stream, mode))
}

int gd_probe_mfma(uint64_t operands, uint64_t out, uint32_t blocks, uint32_t iters, void *hip_stream)
{
    GD_ABI_GUARD(gd::launch_mfma_probe(operands, out, blocks, iters, static_cast<hipStream_t>(hip_stream)))
}

int gd_probe_host_path(gd_pool *pool, int tenant, uint64_t dptr, uint32_t iters, void *hip_stream, int mode, double *ns)
{
    GD_ABI_GUARD(probe_host_path(pool, tenant, dptr, iters, hip_stream, mode, ns))
}

int gd_probe_gather_policy(uint64_t out, uint64_t tab, uint64_t idx, uint64_t n, uint32_t policy, void *hip_stream)
{
    GD_ABI_GUARD(gd::launch_probe_gather_policy(out, tab, idx, n, policy, static_cast<hipStream_t>(hip_stream)))
}

const char *gd_strerror(int status)
{
    switch (status) {
    case GD_OK: return "ok";
    case GD_EINVAL: return "invalid argument";
    case GD_ENOTPOW2: return "partition size is not a power of two of at least 4096";
    case GD_ENOMEM: return "out of pool or partition memory";
    case GD_ERANGE: return "range is not inside the tenant's partition";
    case GD_ENOTENANT: return "no such tenant";
    case GD_EBUSY: return "tenant has live allocations";
    case GD_EHIP: return "HIP call failed";
    case GD_ENOKERNEL: return "unknown kernel or fence mode";
    case GD_ESHAPE: return "operand shape not supported by the kernel";
    default: return "unknown status";
    }
}

int gd_last_hip_error(void) { return gd::g_last_hip_error; }

}  // extern "C"
