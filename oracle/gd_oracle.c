/*
 * CPU oracle for the Guardian fenced-kernel path: kernel semantics.
 *
 * TEST INFRASTRUCTURE ONLY.  Not part of the product; shares no code with the
 * HIP library.  Plain C, one sequential loop per logical element, floating
 * point in fp64, no blocking, no vectorisation, no threads.
 *
 * Timing twin.  Compiled with -fopenmp the same file spreads the loops whose
 * iterations are independent on in-bounds inputs over the host cores (the
 * `GDO_PARALLEL_FOR` lines); that build exists only so that the benchmark can
 * report the oracle's speed on all cores.  Every check uses the sequential build:
 * with out-of-bounds inputs the order of wrapped accesses matters, and the
 * parallel sum adds in another order.
 *
 * Model.  Device memory is a byte array `mem` standing for the address range
 * [pool_base, pool_base + pool_bytes).  A kernel is launched for one tenant and
 * sees only that tenant's row of the partition bounds table (Section 4.2.3):
 * `part_base`, `part_size`.  Every kernel computes the raw address of each
 * access from the pointers the tenant passed, in wrap-around 64-bit
 * arithmetic, then applies the fence to that final effective address, then
 * accesses memory -- the order of Listing 1 (compute address, AND, OR,
 * ld/st) and of Section 4.3's rule for the register+offset addressing mode.
 *
 * Fence rules (`mode`):
 *   0  none      native kernel, Section 4.2.3 (standalone tenant)
 *   1  bitwise   (addr AND mask) OR base, Listing 1 / Section 4.3; the low
 *                log2(width) bits are cleared too (this build's reading: the
 *                paper fences the start address only, and hardware that allows
 *                unaligned accesses needs the whole access inside)
 *   2  modulo    base + ((addr - base) % size), Section 4.4, with the same
 *                width rule: the low log2(width) bits of the offset are cleared
 *                (bases and sizes are multiples of every access width)
 *   3  check     Section 4.4: the access proceeds only if it lies inside the
 *                partition; otherwise the logical thread stops (Section 4.3,
 *                last sentence) and the violation is counted
 *   4  hwcheck   address checking as a GPU's buffer addressing does it (this
 *                build's addition to Section 4.4's list): the access goes to
 *                base + off with off = (addr - base) mod 2^32, low log2(width)
 *                bits cleared, if off + width <= size; otherwise a load reads 0
 *                and a store is dropped, and the thread goes on
 *
 * An access that leaves the simulated pool altogether (possible only in mode 0)
 * is dropped and counted in `escaped`: on a real GPU it would be a fault.
 *
 * Parity status: pinned by tests/test_oracle_kernels.py (textbook NumPy
 * routines on in-bounds inputs, brute-force confinement on tiny pools, the
 * host model's fence).  Values at locations that a kernel's own wrapped stores
 * alias with its own live data are unspecified by the paper: parity unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#define GDO_PRAGMA(x) _Pragma(#x)
#define GDO_PARALLEL_FOR GDO_PRAGMA(omp parallel for schedule(static))
#define GDO_PARALLEL_SUM(v) GDO_PRAGMA(omp parallel for schedule(static) reduction(+ : v))
#define GDO_COUNT(field) do { GDO_PRAGMA(omp atomic) (field)++; } while (0)
int gdo_threads(void) { return omp_get_max_threads(); }
#else
#define GDO_PARALLEL_FOR
#define GDO_PARALLEL_SUM(v)
#define GDO_COUNT(field) ((field)++)
int gdo_threads(void) { return 1; }
#endif

typedef struct {
    uint8_t *mem;          /* simulated device memory                          */
    uint64_t pool_base;    /* device address of mem[0]                         */
    uint64_t pool_bytes;
    uint64_t part_base;    /* launching tenant's partition (bounds table row)  */
    uint64_t part_size;
    int32_t  mode;         /* fence rule, see above                            */
    int32_t  pad;
    uint64_t escaped;      /* out: accesses outside the simulated pool         */
    uint64_t violations;   /* out: accesses refused by mode 3                  */
    uint64_t wrapped;      /* out: accesses whose address the fence changed    */
} gdo_ctx;

/* ---- the fence ----------------------------------------------------------- */

/* Returns 1 and the effective address, or 0 if mode 3 refuses the access. */
static int effective(gdo_ctx *c, uint64_t raw, uint32_t width, uint64_t *eff)
{
    uint64_t base = c->part_base, size = c->part_size;
    switch (c->mode) {
    case 1: {
        uint64_t end  = base + size - 1;           /* highest address          */
        uint64_t mask = end ^ base;                /* Section 4.3 example      */
        mask &= ~(uint64_t)(width - 1);
        *eff = (raw & mask) | base;
        break;
    }
    case 2:
        *eff = base + (((raw - base) % size) & ~(uint64_t)(width - 1));
        break;
    case 3:
        if (raw < base || raw + (width - 1) < raw || raw + (width - 1) > base + size - 1) {
            GDO_COUNT(c->violations);
            return 0;
        }
        *eff = raw;
        break;
    case 4: {
        uint64_t off = ((raw - base) & 0xffffffffu) & ~(uint64_t)(width - 1);
        if (off + width > size) {
            GDO_COUNT(c->violations);
            return 0;
        }
        *eff = base + off;
        break;
    }
    default:
        *eff = raw;
    }
    if (*eff != raw) GDO_COUNT(c->wrapped);
    return 1;
}

uint64_t gdo_fence(uint64_t base, uint64_t size, uint64_t addr, uint32_t width, int32_t mode)
{
    gdo_ctx c;
    memset(&c, 0, sizeof c);
    c.part_base = base; c.part_size = size; c.mode = mode;
    uint64_t eff = 0;
    if (!effective(&c, addr, width, &eff)) return ~(uint64_t)0;
    return eff;
}

void gdo_fence_array(uint64_t base, uint64_t size, const uint64_t *addr, uint64_t n,
                     uint32_t width, int32_t mode, uint64_t *out)
{
    for (uint64_t i = 0; i < n; i++) out[i] = gdo_fence(base, size, addr[i], width, mode);
}

/* ---- memory accesses ------------------------------------------------------ */

/* 1 = done, 0 = the logical thread must stop (mode 3).  A refused access reads 0;
 * in mode 4 the thread goes on with that value. */
static int ld(gdo_ctx *c, uint64_t raw, uint32_t width, void *dst)
{
    uint64_t a;
    memset(dst, 0, width);
    if (!effective(c, raw, width, &a)) return c->mode == 4;
    if (a < c->pool_base || a - c->pool_base > c->pool_bytes - width || c->pool_bytes < width) {
        GDO_COUNT(c->escaped);
        return 1;
    }
    memcpy(dst, c->mem + (a - c->pool_base), width);
    return 1;
}

static int st(gdo_ctx *c, uint64_t raw, uint32_t width, const void *src)
{
    uint64_t a;
    if (!effective(c, raw, width, &a)) return c->mode == 4;      /* mode 4: dropped, the thread goes on */
    if (a < c->pool_base || a - c->pool_base > c->pool_bytes - width || c->pool_bytes < width) {
        GDO_COUNT(c->escaped);
        return 1;
    }
    memcpy(c->mem + (a - c->pool_base), src, width);
    return 1;
}

/* ---- bfloat16 ------------------------------------------------------------- */

static double bf16_to_double(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* Round a double to the nearest bfloat16 (8 significant bits, float's exponent
 * range), ties to even, in one rounding step. */
static uint16_t double_to_bf16(double x)
{
    float f;
    uint32_t u;
    if (isnan(x)) return 0x7fc0;
    if (isinf(x) || x == 0.0) {
        f = (float)x;
    } else {
        int e;
        frexp(x, &e);                      /* |x| = m * 2^e, 0.5 <= m < 1       */
        int ulp = e - 8;                   /* 8 significant bits                */
        if (ulp < -133) ulp = -133;        /* bfloat16 subnormal spacing        */
        double r = ldexp(nearbyint(ldexp(x, -ulp)), ulp);   /* ties to even    */
        f = (float)r;                      /* exact, or overflows to infinity   */
    }
    memcpy(&u, &f, 4);
    return (uint16_t)(u >> 16);
}

uint16_t gdo_double_to_bf16(double x) { return double_to_bf16(x); }
double   gdo_bf16_to_double(uint16_t h) { return bf16_to_double(h); }

/* ---- kernels --------------------------------------------------------------
 * Each loop body is one logical thread.  `continue` = that thread stops.     */

/* Listing 1's sample kernel as the text of Section 4.3 describes it:
 * A[i] = j for every thread i. */
void gdo_store_tid(gdo_ctx *c, uint64_t A, uint32_t j, uint64_t n)
{
    for (uint64_t i = 0; i < n; i++) {
        if (!st(c, A + 4 * i, 4, &j)) continue;
    }
}

/* Probe: out[i] = fence_width(in[i]); the loads and stores of the probe itself
 * are 8-byte tenant accesses and are fenced like any other. */
void gdo_fence_addrs(gdo_ctx *c, uint64_t out, uint64_t in, uint32_t width, uint64_t n)
{
    for (uint64_t i = 0; i < n; i++) {
        uint64_t a, f;
        if (!ld(c, in + 8 * i, 8, &a)) continue;
        if (!effective(c, a, width, &f)) f = ~(uint64_t)0;
        if (!st(c, out + 8 * i, 8, &f)) continue;
    }
}

/* STREAM copy: a[i] = b[i], 4-byte elements moved bit for bit. */
void gdo_copy(gdo_ctx *c, uint64_t a, uint64_t b, uint64_t n)
{
    GDO_PARALLEL_FOR
    for (uint64_t i = 0; i < n; i++) {
        uint32_t v;
        if (!ld(c, b + 4 * i, 4, &v)) continue;
        if (!st(c, a + 4 * i, 4, &v)) continue;
    }
}

/* STREAM triad: a[i] = b[i] + s * c[i]. */
void gdo_triad(gdo_ctx *c, uint64_t a, uint64_t b, uint64_t cc, double s, uint64_t n)
{
    GDO_PARALLEL_FOR
    for (uint64_t i = 0; i < n; i++) {
        float vb, vc, r;
        if (!ld(c, b + 4 * i, 4, &vb)) continue;
        if (!ld(c, cc + 4 * i, 4, &vc)) continue;
        r = (float)((double)vb + s * (double)vc);
        if (!st(c, a + 4 * i, 4, &r)) continue;
    }
}

/* Indexed saxpy: o = off[i] (signed 32-bit element offset);
 * y[o] = alpha * x[o] + y[o]. */
void gdo_saxpy_idx(gdo_ctx *c, uint64_t x, uint64_t y, uint64_t off, double alpha, uint64_t n)
{
    for (uint64_t i = 0; i < n; i++) {
        int32_t o;
        float vx, vy, r;
        if (!ld(c, off + 4 * i, 4, &o)) continue;
        uint64_t byte_off = (uint64_t)((int64_t)o * 4);
        if (!ld(c, x + byte_off, 4, &vx)) continue;
        if (!ld(c, y + byte_off, 4, &vy)) continue;
        r = (float)(alpha * (double)vx + (double)vy);
        if (!st(c, y + byte_off, 4, &r)) continue;
    }
}

/* Pointer chase (the dependent-access chain behind the latency model of Section 4.4, Figure 5, and the
 * cache-resident regime of Section 7.4): logical thread t starts at index start + t * lane_step and replaces
 * its index `steps` times by the 4-byte table entry it points at, every access through the rule like any
 * other; out[t] receives the last index.  Thread 0 then stores two 8-byte counters at clk (elapsed time on
 * the device: what they hold is not part of the result; the oracle stores zeros). */
void gdo_chase(gdo_ctx *c, uint64_t out, uint64_t clk, uint64_t tab, uint64_t steps, uint32_t start,
               uint32_t lane_step, uint32_t threads)
{
    for (uint32_t t = 0; t < threads; t++) {
        uint32_t idx = start + t * lane_step;
        uint64_t zero = 0, s;
        int alive = 1;
        for (s = 0; s < steps && alive; s++)
            alive = ld(c, tab + 4 * (uint64_t)idx, 4, &idx);
        if (!alive) continue;
        if (!st(c, out + 4 * (uint64_t)t, 4, &idx)) continue;
        if (t != 0) continue;
        if (!st(c, clk, 8, &zero)) continue;
        if (!st(c, clk + 8, 8, &zero)) continue;
    }
}

/* Gather of 4-byte values with 64-bit indices: out[i] = tab[idx[i]]. */
void gdo_gather32_i64(gdo_ctx *c, uint64_t out, uint64_t tab, uint64_t idx, uint64_t n)
{
    GDO_PARALLEL_FOR
    for (uint64_t i = 0; i < n; i++) {
        uint64_t k;
        uint32_t v;
        if (!ld(c, idx + 8 * i, 8, &k)) continue;
        if (!ld(c, tab + 4 * k, 4, &v)) continue;
        if (!st(c, out + 4 * i, 4, &v)) continue;
    }
}

/* Gather of 4-byte values with signed 32-bit indices: out[i] = tab[idx[i]]. */
void gdo_gather32_i32(gdo_ctx *c, uint64_t out, uint64_t tab, uint64_t idx, uint64_t n)
{
    GDO_PARALLEL_FOR
    for (uint64_t i = 0; i < n; i++) {
        int32_t k;
        uint32_t v;
        if (!ld(c, idx + 4 * i, 4, &k)) continue;
        if (!ld(c, tab + (uint64_t)((int64_t)k * 4), 4, &v)) continue;
        if (!st(c, out + 4 * i, 4, &v)) continue;
    }
}

/* Scatter of fp32 values with 64-bit indices: dst[idx[i]] = scale * src[i]. */
void gdo_scatter_f32_i64(gdo_ctx *c, uint64_t dst, uint64_t src, uint64_t idx, double scale, uint64_t n)
{
    GDO_PARALLEL_FOR
    for (uint64_t i = 0; i < n; i++) {
        uint64_t k;
        float v, r;
        if (!ld(c, idx + 8 * i, 8, &k)) continue;
        if (!ld(c, src + 4 * i, 4, &v)) continue;
        r = (float)(scale * (double)v);
        if (!st(c, dst + 4 * k, 4, &r)) continue;
    }
}

/* Sum of n fp32 values, accumulated in fp64 in index order, written as one fp32. */
void gdo_sum_f32(gdo_ctx *c, uint64_t out, uint64_t in, uint64_t n)
{
    double acc = 0.0;
    GDO_PARALLEL_SUM(acc)
    for (uint64_t i = 0; i < n; i++) {
        float v;
        if (!ld(c, in + 4 * i, 4, &v)) continue;
        acc += (double)v;
    }
    float r = (float)acc;
    st(c, out, 4, &r);
}

/* The same sum returned in fp64 (what the fp32 result is compared against). */
double gdo_sum_f32_exact(gdo_ctx *c, uint64_t in, uint64_t n)
{
    double acc = 0.0;
    GDO_PARALLEL_SUM(acc)
    for (uint64_t i = 0; i < n; i++) {
        float v;
        if (!ld(c, in + 4 * i, 4, &v)) continue;
        acc += (double)v;
    }
    return acc;
}

/* Row-wise RMS normalisation of a row-major rows x cols bfloat16 matrix:
 * y[r,j] = bf16( x[r,j] / sqrt(mean_j(x[r,j]^2) + eps) * g[j] ).
 *
 * Logical thread (r, j) produces y[r,j]: it reads all of row r (the mean needs
 * every value), then g[j], then stores.  Under address checking (mode 3) a
 * thread returns at its first refused access (Section 4.3, last sentence;
 * Section 4.4), so a refused access to x[r,k] stops all `cols` threads of the row
 * -- each of them meets it -- and each counts one violation; a refused g[j] or
 * y[r,j] stops that one thread. */
void gdo_rmsnorm_bf16(gdo_ctx *c, uint64_t y, uint64_t x, uint64_t g,
                      uint64_t rows, uint64_t cols, double eps)
{
    GDO_PARALLEL_FOR
    for (uint64_t r = 0; r < rows; r++) {
        double ss = 0.0;
        int row_read = 1;
        for (uint64_t j = 0; j < cols; j++) {
            uint16_t h;
            if (!ld(c, x + 2 * (r * cols + j), 2, &h)) { row_read = 0; break; }
            double v = bf16_to_double(h);
            ss += v * v;
        }
        if (!row_read) {
            c->violations += cols - 1;     /* the other threads of the row stop at the same access */
            continue;
        }
        double inv = 1.0 / sqrt(ss / (double)cols + eps);
        for (uint64_t j = 0; j < cols; j++) {
            uint16_t h, hg, o;
            if (!ld(c, x + 2 * (r * cols + j), 2, &h)) continue;    /* passed above */
            if (!ld(c, g + 2 * j, 2, &hg)) continue;
            o = double_to_bf16(bf16_to_double(h) * inv * bf16_to_double(hg));
            if (!st(c, y + 2 * (r * cols + j), 2, &o)) continue;
        }
    }
}

/* C = A * B on bfloat16 operands, fp64 accumulation, bfloat16 result.
 * A is row-major M x K.  B is row-major K x N if b_is_nk == 0, or stored as
 * N x K (each column of B contiguous) if b_is_nk != 0.  C is row-major M x N.
 * Only rows [m0, m1) and columns [n0, n1) of C are computed, so that a test
 * can ask for a slab or single entries of a large product.
 *
 * Logical thread (m, n) produces C[m,n] from row m of A and column n of B; under
 * address checking (mode 3) it returns at its first refused access and stores
 * nothing (one violation per stopped thread). */
void gdo_gemm_bf16(gdo_ctx *c, uint64_t C, uint64_t A, uint64_t B,
                   uint64_t M, uint64_t N, uint64_t K, int32_t b_is_nk,
                   uint64_t m0, uint64_t m1, uint64_t n0, uint64_t n1)
{
    (void)M;
    GDO_PARALLEL_FOR
    for (uint64_t m = m0; m < m1; m++) {
        for (uint64_t n = n0; n < n1; n++) {
            double acc = 0.0;
            int stopped = 0;
            for (uint64_t k = 0; k < K; k++) {
                uint16_t ha, hb;
                if (!ld(c, A + 2 * (m * K + k), 2, &ha)) { stopped = 1; break; }
                if (!ld(c, B + 2 * (b_is_nk ? n * K + k : k * N + n), 2, &hb)) { stopped = 1; break; }
                acc += bf16_to_double(ha) * bf16_to_double(hb);
            }
            if (stopped) continue;
            uint16_t o = double_to_bf16(acc);
            if (!st(c, C + 2 * (m * N + n), 2, &o)) continue;
        }
    }
}

/* The same dot product returned in fp64 for one entry of C (no store). */
double gdo_gemm_bf16_entry(gdo_ctx *c, uint64_t A, uint64_t B, uint64_t N, uint64_t K,
                           int32_t b_is_nk, uint64_t m, uint64_t n)
{
    double acc = 0.0;
    for (uint64_t k = 0; k < K; k++) {
        uint16_t ha, hb;
        ld(c, A + 2 * (m * K + k), 2, &ha);
        ld(c, B + 2 * (b_is_nk ? n * K + k : k * N + n), 2, &hb);
        acc += bf16_to_double(ha) * bf16_to_double(hb);
    }
    return acc;
}
