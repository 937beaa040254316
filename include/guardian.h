/*
 * guardian.h -- C ABI of libguardian: fenced GPU kernels over a partitioned pool.
 *
 * One GPU address range (the pool) is split into one contiguous, power-of-two
 * sized, size-aligned partition per tenant (paper Sections 1, 4.2.1, 4.4).
 * Host-initiated copies are range-checked against the partition bounds table
 * (Section 4.2.2).  Every kernel launched through gd_launch_fenced receives
 * the launching tenant's base and mask as two extra parameters and applies
 *     addr = (addr AND mask) OR base
 * to the final effective address of every global load and store (Listing 1,
 * Section 4.3), so an out-of-partition access wraps into the tenant's own
 * partition and an in-partition access is unchanged.
 *
 * Conventions.  Device addresses cross this ABI as uint64_t.  The library
 * never dereferences pool memory on the host, so every call that launches no
 * kernel (all but gd_launch_fenced, gd_sum_f32_noalloc and the gd_probe_*
 * measurement aids) also works with made-up addresses and without a GPU.  All
 * functions return a gd_status; on error, out-parameters are left untouched.
 * Nothing aborts, nothing throws across the ABI (host allocation failure is
 * reported as GD_ENOMEM).  A pool is protected by one mutex: calls on the same
 * pool from several threads are serialised.
 */
#ifndef GUARDIAN_H
#define GUARDIAN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gd_pool gd_pool;

typedef enum {
    GD_OK = 0,
    GD_EINVAL = 1,     /* null pointer, zero size, bad alignment argument, bad args size */
    GD_ENOTPOW2 = 2,   /* partition size is not a power of two of at least GD_MIN_PARTITION */
    GD_ENOMEM = 3,     /* no room in the pool / in the partition */
    GD_ERANGE = 4,     /* range not inside the tenant's partition */
    GD_ENOTENANT = 5,  /* tenant number not attached */
    GD_EBUSY = 6,      /* tenant still has live allocations */
    GD_EHIP = 7,       /* a HIP call failed; see gd_last_hip_error() */
    GD_ENOKERNEL = 8,  /* unknown kernel id or fence mode not built for it */
    GD_ESHAPE = 9      /* operand shape outside what the kernel supports */
} gd_status;

#define GD_MIN_PARTITION 4096u  /* bytes */
#define GD_GRANULE 256u         /* allocation granule and minimum alignment, bytes */

/* Fence rule applied by the launched kernel (Section 4.4 lists the choices). */
typedef enum {
    GD_FENCE_NONE = 0,     /* native kernel: tenant runs alone, protection off (Section 4.2.3) */
    GD_FENCE_BITWISE = 1,  /* AND with mask, OR with base (Listing 1); needs size-aligned pow2 partitions */
    GD_FENCE_MODULO = 2,   /* base + (addr - base) % size (Section 4.4); any size, any alignment */
    GD_FENCE_CHECK = 3,    /* compare against base/end; an offending logical thread stops and is counted
                              (Sections 4.3, 4.4).  A logical thread is the computation of one output
                              element: in RMSNorm and GEMM it reads a whole operand row (and column), so
                              an operand row that is not wholly inside stops every thread that needs it */
    GD_FENCE_HWCHECK = 4   /* address checking by the memory pipeline (an addition: the GPU's buffer
                              instructions compare every access with the partition's size, Section 4.4's
                              conditional check without instructions): offset = lo32(addr - base) with
                              the low log2(width) bits cleared; an access outside reads 0 / is dropped,
                              the thread goes on, nothing is counted.  Partitions below 4 GiB, any size
                              and alignment (GD_ESHAPE otherwise) */
} gd_fence_mode;

/* ---- pool and partition bounds table (Section 4.2.1) ---------------------- */

/* Carve [dev_base, dev_base + dev_bytes) into n_tenants partitions of
 * part_bytes[i] bytes, tenant i = index i.  The caller owns the memory (it must
 * stay allocated until gd_pool_destroy) and the library only borrows the range.
 * Each size must be a power of two >= GD_MIN_PARTITION (else GD_ENOTPOW2).
 * Placement: tenants by decreasing size (ties by index), each at the lowest
 * size-aligned address of the pool that is still free; GD_ENOMEM if one does
 * not fit (a dev_base that is not aligned to the largest size costs slack).
 * n_tenants may be 0 (part_bytes may then be NULL). */
int gd_pool_create(uint64_t dev_base, uint64_t dev_bytes, const uint64_t *part_bytes,
                   int n_tenants, gd_pool **out);

/* The same for partitions of ARBITRARY size (Section 4.4: the modulo fence and
 * address checking need neither power-of-two sizes nor alignment).  Sizes must be
 * multiples of GD_GRANULE and at least GD_MIN_PARTITION (else GD_ENOTPOW2);
 * partitions are placed in tenant order, each at the lowest GD_GRANULE-aligned
 * free address.  Kernels on such a pool can only be launched with
 * GD_FENCE_MODULO, GD_FENCE_CHECK, GD_FENCE_HWCHECK or GD_FENCE_NONE
 * (GD_FENCE_BITWISE: GD_EINVAL);
 * gd_tenant_attach on it follows the same placement rule. */
int gd_pool_create_flex(uint64_t dev_base, uint64_t dev_bytes, const uint64_t *part_bytes,
                        int n_tenants, gd_pool **out);

/* Address checking reports violations in a per-tenant uint64 counter (one per
 * tenant number, `slots` of them) at device address `dev_counters`.  The array
 * is owned by the caller in the manager's role: it must lie outside the pool (else
 * GD_EINVAL), be 8-byte aligned and zeroed by the caller.  Required before any
 * GD_FENCE_CHECK launch. */
int gd_pool_set_fault_counters(gd_pool *pool, uint64_t dev_counters, int slots);

/* Frees host metadata only. */
int gd_pool_destroy(gd_pool *pool);

/* Re-carving while other tenants keep running (Section 2.2, point (1): partitions
 * sized per application, no reset).  attach places a new partition by the same
 * rule and returns the lowest unused tenant number; detach releases a partition
 * (GD_EBUSY while the tenant has live allocations).  Other rows never move.
 * The library cannot see kernels in flight: the caller must drain the tenant's
 * stream(s) before gd_tenant_detach, or a kernel still queued for the old
 * tenant can write into a range that gd_tenant_attach has handed to a new one. */
int gd_tenant_attach(gd_pool *pool, uint64_t bytes, int *tenant_out);
int gd_tenant_detach(gd_pool *pool, int tenant);

/* One row of the bounds table; mask = size - 1 (Section 4.3 worked example).
 * Any of base/size/mask may be NULL. */
int gd_partition_info(const gd_pool *pool, int tenant, uint64_t *base, uint64_t *size,
                      uint64_t *mask);

/* ---- allocation inside a partition (Section 4.2.1) ------------------------- */

/* Address-ordered first fit inside the tenant's partition.  bytes is rounded
 * up to GD_GRANULE; align must be a power of two (values below GD_GRANULE are
 * raised to it).  bytes == 0 or a bad align: GD_EINVAL; no room: GD_ENOMEM.
 * Bookkeeping lives on the host only, never inside the partition. */
int gd_alloc(gd_pool *pool, int tenant, uint64_t bytes, uint64_t align, uint64_t *dptr_out);

/* dptr must be the start of a live allocation of that tenant (else GD_EINVAL). */
int gd_free(gd_pool *pool, int tenant, uint64_t dptr);

/* ---- transfer range check (Section 4.2.2) ----------------------------------- */

/* GD_OK iff [dptr, dptr + bytes) lies inside the tenant's partition, else
 * GD_ERANGE.  Partition bounds only, not allocation bounds (Section 5,
 * "Buffer overflow").  Performs no copy: the caller copies on GD_OK.  Call it
 * once per device pointer of a memcpy/memset (twice for device-to-device). */
int gd_check_copy(const gd_pool *pool, int tenant, uint64_t dptr, uint64_t bytes);

/* ---- kernels (Section 4.2.3: lookup of the sandboxed kernel, two extra
 *      parameters, launch on the tenant's stream) ----------------------------- */

typedef enum {
    GD_K_STORE_TID = 0,    /* A[i] = j                         (Listing 1's sample kernel) */
    GD_K_FENCE_ADDRS = 1,  /* out[i] = fence_width(in[i])      (probe of the device fence) */
    GD_K_COPY = 2,         /* a[i] = b[i], 4-byte elements     (STREAM copy) */
    GD_K_TRIAD = 3,        /* a[i] = b[i] + s*c[i], fp32       (STREAM triad) */
    GD_K_SAXPY_IDX = 4,    /* o = off[i]; y[o] = alpha*x[o] + y[o], fp32, int32 offsets */
    GD_K_GATHER32_I64 = 5, /* out[i] = tab[idx[i]], 4-byte values, int64 indices */
    GD_K_SCATTER_F32_I64 = 6, /* dst[idx[i]] = scale*src[i], fp32, int64 indices */
    GD_K_GATHER32_I32 = 7, /* out[i] = tab[idx[i]], 4-byte values, int32 indices */
    GD_K_SUM_F32 = 8,      /* out[0] = sum of in[0..n), fp32 */
    GD_K_RMSNORM_BF16 = 9, /* y[r,:] = x[r,:] / sqrt(mean(x[r,:]^2) + eps) * g, bf16 in/out, fp32 math */
    GD_K_GEMM_BF16 = 10,   /* C = A*B, bf16 in/out, fp32 accumulate on MFMA */
    GD_K_CHASE = 11,       /* i = tab[i], steps times, per logical thread (latency of a fenced access: Section 4.4, Figure 5) */
    GD_K_COUNT = 12
} gd_kernel_id;

/* Argument blocks.  Pointers are tenant-supplied device addresses; they are NOT
 * validated on the host -- the fence is the protection, as in the paper.  An
 * element address is ptr + elem_bytes*index in wrap-around 64-bit arithmetic,
 * and the fence is applied to that final address. */
typedef struct { uint64_t A; uint64_t n; uint32_t j; uint32_t pad; } gd_args_store_tid;
typedef struct { uint64_t out; uint64_t in; uint64_t n; uint32_t width; uint32_t pad; } gd_args_fence_addrs;
typedef struct { uint64_t a; uint64_t b; uint64_t n; } gd_args_copy;
/* repeat: the whole operation is performed max(repeat, 1) times (same result; lets a caller keep a
 * small working set cache resident inside one launch, Section 7.4's regime). */
typedef struct { uint64_t a; uint64_t b; uint64_t c; uint64_t n; float s; uint32_t repeat; } gd_args_triad;
typedef struct { uint64_t x; uint64_t y; uint64_t off; uint64_t n; float alpha; uint32_t pad; } gd_args_saxpy_idx;
typedef struct { uint64_t out; uint64_t tab; uint64_t idx; uint64_t n; } gd_args_gather;
typedef struct { uint64_t dst; uint64_t src; uint64_t idx; uint64_t n; float scale; uint32_t pad; } gd_args_scatter;
/* partials: tenant workspace of GD_SUM_WORKSPACE bytes, contents unspecified afterwards. */
typedef struct { uint64_t out; uint64_t in; uint64_t partials; uint64_t n; } gd_args_sum;
typedef struct { uint64_t y; uint64_t x; uint64_t g; uint32_t rows; uint32_t cols; float eps; uint32_t pad; } gd_args_rmsnorm;
/* A row-major M x K.  B row-major K x N (b_is_nk == 0) or stored N x K, K contiguous
 * (b_is_nk != 0).  C row-major M x N. */
typedef struct { uint64_t C; uint64_t A; uint64_t B; uint32_t M; uint32_t N; uint32_t K; uint32_t b_is_nk; } gd_args_gemm;

/* Pointer chase: logical thread t < threads (at most 64: one wavefront) starts at index start + t*lane_step and
 * replaces its index `steps` times by the uint32 entry tab[index]; every access is fenced like any other, and
 * each depends on the one before, so steps / elapsed time is the latency of one fenced access (Section 4.4's
 * model: cycles of the fence against cycles of the access, Figure 5; Section 7.4's cache-resident regime is
 * chosen by the footprint of the entries the chain visits).  out[t] (uint32) receives thread t's last index.
 * Thread 0 then stores two uint64 at clk: the shader-clock cycles and the ticks of the constant 100 MHz
 * counter that its chain took (measurements, not results: no other call defines their value).  Fixed launch
 * shape (one wavefront); threads == 0 or > 64: GD_ESHAPE. */
typedef struct { uint64_t out; uint64_t clk; uint64_t tab; uint64_t steps; uint32_t start; uint32_t lane_step; uint32_t threads; uint32_t pad; } gd_args_chase;

#define GD_SUM_WORKSPACE 16384u /* bytes */

/* Launch kernel_id for a tenant, asynchronously, on the caller-owned HIP stream
 * (hipStream_t passed as void*; NULL = the null stream).  The library looks the
 * kernel up, appends the tenant's {base, mask} from the bounds table to a copy
 * of *args and launches the variant built for `mode`.  args_bytes must equal
 * the size of the kernel's argument block (GD_EINVAL otherwise).
 * grid/block: NULL lets the library choose the launch shape it was tuned for.
 * Element-wise kernels (ids 0..7) also accept a caller-chosen 1-D shape
 * (grid[0], block[0]; block[0] a multiple of 64 up to 1024) and loop over
 * their input; the others have a fixed shape and return GD_EINVAL for non-NULL.
 * Shapes a kernel cannot run are refused with GD_ESHAPE before any launch.
 * HIP failures give GD_EHIP. */
int gd_launch_fenced(gd_pool *pool, int tenant, int kernel_id, const void *args,
                     size_t args_bytes, const uint32_t grid[3], const uint32_t block[3],
                     void *hip_stream, int mode);

/* For callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the fp32 sum of
 * GD_K_SUM_F32 without a workspace argument.  The per-workgroup partial sums go
 * to a file-scope device array of the library (GD_SUM_NOALLOC_SCRATCH bytes, held
 * by every GPU the library runs on until the process ends) instead of tenant
 * memory; that array is manager-owned, outside every pool, and its accesses are
 * not fenced.  `out` and `in` are tenant addresses and are fenced as in
 * gd_launch_fenced with the same `mode`; the result equals that of GD_K_SUM_F32
 * bit for bit.  The call allocates nothing and synchronises nothing.  The first
 * call on a device looks the array's address up (hipGetSymbolAddress): make one
 * call outside any capture first.  n above GD_SUM_NOALLOC_MAX_N: GD_ESHAPE,
 * nothing launched.  All calls on one GPU share the one array: calls that can
 * overlap in time on the same GPU (different streams without an ordering
 * between them) race on it and must be serialised by the caller. */
#define GD_SUM_NOALLOC_MAX_N (1ull << 32)   /* elements */
#define GD_SUM_NOALLOC_SCRATCH 8192u        /* bytes */
int gd_sum_f32_noalloc(gd_pool *pool, int tenant, uint64_t out, uint64_t in, uint64_t n,
                       void *hip_stream, int mode);

/* Kernel registry (the analogue of the paper's pointerToSymbol map). */
int gd_kernel_count(void);
const char *gd_kernel_name(int kernel_id);         /* NULL if unknown */
size_t gd_kernel_args_bytes(int kernel_id);        /* 0 if unknown */

/* ---- helpers ----------------------------------------------------------------- */

/* Host twin of the device fence for mode BITWISE/MODULO (Listing 1; Section 4.4):
 * the address a `width`-byte access (1, 2, 4, 8 or 16) to addr is redirected to.
 * For BITWISE the low log2(width) bits are cleared as well, so that the whole
 * access lies inside the partition.  Returns UINT64_MAX for bad arguments or,
 * in mode CHECK or HWCHECK, for an access that is not inside. */
uint64_t gd_fence_host(uint64_t base, uint64_t size, uint64_t addr, uint32_t width, int mode);

/* Measurement aid, not part of the fenced path (no pool, no tenant, no fence): a
 * kernel that does nothing but the GEMM's matrix instructions (v_mfma_f32_16x16x32_bf16,
 * 64 per wavefront and iteration, 256 accumulators per lane) on operands it holds in
 * registers.  Its rate on N(0,1) operands is what the matrix pipe sustains under the
 * chip's power limit -- the ceiling the GEMM of Section-4-style fenced tile loads is
 * measured against.  operands: device address of 64 KiB of bfloat16 values (16-byte
 * aligned; 16 fragments x 256 threads x 8 values); out: device address of blocks*256
 * floats (a checksum per thread, so that the loop cannot be optimised away).  Both are
 * caller-owned plain device memory.  flop per launch = blocks * 4 * iters * 2^20. */
int gd_probe_mfma(uint64_t operands, uint64_t out, uint32_t blocks, uint32_t iters, void *hip_stream);

/* Measurement aid, not part of the fenced path (no pool, no tenant, no fence):
 * out[i] = tab[idx[i]] for 4-byte values and 64-bit indices, the table load carrying
 * the cache-policy bits `policy` (bit 0 = sc0, bit 1 = sc1, bit 2 = nt).  The caller
 * owns all three arrays (plain device memory; out and idx 16-byte aligned, n a multiple
 * of 4) and guarantees that every index addresses the table and that the table is
 * smaller than 4 GiB.  bench.py times the eight combinations and, under rocprofv3,
 * reads the bytes each fetches past the L2. */
int gd_probe_gather_policy(uint64_t out, uint64_t tab, uint64_t idx, uint64_t n, uint32_t policy,
                           void *hip_stream);

/* Measurement aid: what the fenced launch path costs on the host, per call, timed
 * inside the library (no language binding in the figures) -- the analogue of the
 * paper's Table 5 (Section 7.6: kernel lookup and parameter augmentation against the
 * launch call itself).  Uses GD_K_STORE_TID on 64 elements at `dptr`, a device
 * address the caller has allocated in `tenant`'s partition (256 bytes are written,
 * fenced under `mode`).  ns[0]: gd_launch_fenced up to the launch (lookup, bounds-table
 * row, parameter augmentation; an n = 0 launch returns there); ns[1]: gd_launch_fenced
 * including the launch; ns[2]: the bare HIP launch call of the same kernel with
 * arguments prepared once.  Each is the mean over `iters` calls (1 .. 2^20) on
 * `hip_stream`, which is synchronised before and after each of the three loops: this
 * call blocks, unlike every other entry point.  ns is host memory, 3 doubles,
 * untouched on error. */
int gd_probe_host_path(gd_pool *pool, int tenant, uint64_t dptr, uint32_t iters, void *hip_stream, int mode,
                       double *ns);

const char *gd_strerror(int status);
int gd_last_hip_error(void);   /* hipError_t of the last failed HIP call on this thread */

#ifdef __cplusplus
}
#endif
#endif /* GUARDIAN_H */
