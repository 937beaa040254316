// Reductions: fp32 sum of a contiguous array (two passes: per-workgroup partial
// sums into the tenant's workspace, then one workgroup adds the partials) and
// row-wise RMS normalisation of a bf16 matrix (one workgroup per row, the row
// kept in registers between the sum of squares and the scaling).  Wavefront
// reductions use cross-lane shuffles, workgroup reductions a few LDS words; LDS
// is not tenant-addressable and is not fenced.  Every global access, including
// those to the workspace, carries the fence on its final address.
#include <mutex>

#include "launchers.hpp"

namespace gd {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int WG = 256;
constexpr int WAVES = WG / 64;

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

// Sum over a workgroup of NW wavefronts; the result is valid in every thread.
template <int NW = WAVES, typename T>
__device__ __forceinline__ T block_sum(T v, T *lds)
{
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
    __syncthreads();
    T r = lds[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) r += lds[w];
    __syncthreads();
    return r;
}

// ---- sum, pass 1: partials[block] = sum of this block's tiles ---------------------
constexpr int SUM_UNROLL = 4;
constexpr int SUM_TILE = 1024;         // bytes one wavefront covers with one 16-byte vector per lane

// OWN_WS: `partials` is the library's own device array (not tenant-addressable, like the
// fault counters), so the accesses to it are not fenced.
template <int V, bool OWN_WS = false>
__global__ __launch_bounds__(WG) void k_sum_partial(gd_args_sum p, FenceArgs fa)
{
    const Fence<V> F(fa);
    __shared__ float lds[WAVES];
    float acc = 0.0f;
    if ((p.in & 15) == 0) {
        const uint64_t n4 = p.n >> 2;
        const uint64_t tile = (uint64_t)WG * SUM_UNROLL;
        f32x4 a4 = {0.0f, 0.0f, 0.0f, 0.0f};
        const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        const uint32_t lane_off = Fence<V>::template tile_lane_offset<SUM_TILE>(16 * threadIdx.x);
        const bool whole = F.whole_run(p.in, 16 * n4);     // the input is mapped to one contiguous range (wholly inside, if checked)
        const uint64_t f_in = F.scalar_fence(p.in);        // fenced first byte; used only if `whole`
        for (uint64_t t0 = blockIdx.x * tile; t0 < n4; t0 += gridDim.x * tile) {
            const uint64_t i0 = t0 + threadIdx.x;
            if (whole && t0 + tile <= n4) {
                // Full tiles: each of a wavefront's SUM_UNROLL accesses covers one contiguous 1 KiB at
                // "fenced start + offset".
                f32x4 v[SUM_UNROLL];
#pragma unroll
                for (int u = 0; u < SUM_UNROLL; ++u)
                    v[u] = F.template ld_tile16<f32x4, true>(f_in + 16 * (t0 + (uint64_t)u * WG + 64 * wave), lane_off);
                static_assert(SUM_UNROLL == 4, "the wait below names four vectors");
                F.tile_wait(v[0], v[1]);
                F.tile_wait(v[2], v[3]);
#pragma unroll
                for (int u = 0; u < SUM_UNROLL; ++u) a4 += v[u];
            } else if (!F.CHECKED && t0 + tile <= n4) {
                f32x4 v[SUM_UNROLL];
#pragma unroll
                for (int u = 0; u < SUM_UNROLL; ++u) v[u] = F.template ld<f32x4, true>(p.in + 16 * (i0 + (uint64_t)u * WG));
#pragma unroll
                for (int u = 0; u < SUM_UNROLL; ++u) a4 += v[u];
            } else {
#pragma unroll
                for (int u = 0; u < SUM_UNROLL; ++u) {
                    const uint64_t i = i0 + (uint64_t)u * WG;
                    if (i >= n4) continue;
                    if (F.template inside<16>(p.in + 16 * i)) {
                        a4 += F.template ld<f32x4, true>(p.in + 16 * i);
                    } else {                       // address checking: element by element, offenders contribute nothing
                        for (int e = 0; e < 4; ++e) {
                            if (F.template inside<4>(p.in + 16 * i + 4 * e)) a4[e] += F.template ld<float>(p.in + 16 * i + 4 * e);
                            else F.fault();
                        }
                    }
                }
            }
        }
        acc = (a4[0] + a4[1]) + (a4[2] + a4[3]);
        if (blockIdx.x == 0 && threadIdx.x < (p.n & 3)) {
            const uint64_t a = p.in + 4 * (4 * n4 + threadIdx.x);
            if (F.template inside<4>(a)) acc += F.template ld<float>(a);
            else F.fault();
        }
    } else {
        const uint64_t stride = (uint64_t)gridDim.x * WG;
        for (uint64_t i = (uint64_t)blockIdx.x * WG + threadIdx.x; i < p.n; i += stride) {
            if (F.template inside<4>(p.in + 4 * i)) acc += F.template ld<float>(p.in + 4 * i);
            else F.fault();
        }
    }
    const float total = block_sum(acc, lds);
    // the workspace and the result are tenant memory too; a refused access to them is counted and dropped
    if (threadIdx.x == 0) {
        const uint64_t a = p.partials + 4 * (uint64_t)blockIdx.x;
        if constexpr (OWN_WS) *(GD_GLOBAL float *)a = total;
        else if (F.template inside<4>(a)) F.template st<float>(a, total);
        else F.fault();
    }
}

// ---- sum, pass 2: out[0] = sum of the partials (added in fp64) ---------------------
// One workgroup wide enough that every thread has at most FIN_PER partials, fetched before any is used: the pass
// is one memory latency long.  (Its 4.4 us are mostly what any dependent one-workgroup launch costs; against 256
// threads walking eight partials each the pair of launches gained about 1 %.)
constexpr int FIN_WG = 1024;
constexpr int FIN_PER = 2;

template <int V, bool OWN_WS = false>
__global__ __launch_bounds__(FIN_WG) void k_sum_final(gd_args_sum p, uint32_t n_partials, FenceArgs fa)
{
    const Fence<V> F(fa);
    __shared__ double lds[FIN_WG / 64];
    float v[FIN_PER];
#pragma unroll
    for (int u = 0; u < FIN_PER; ++u) {
        const uint32_t i = threadIdx.x + u * FIN_WG;
        const uint64_t a = p.partials + 4 * (uint64_t)i;
        v[u] = 0.0f;
        if (i < n_partials) {
            if constexpr (OWN_WS) v[u] = *(const GD_GLOBAL float *)a;
            else if (F.template inside<4>(a)) v[u] = F.template ld<float>(a);
            else F.fault();
        }
    }
    double acc = 0.0;
#pragma unroll
    for (int u = 0; u < FIN_PER; ++u) acc += (double)v[u];
    const double total = block_sum<FIN_WG / 64>(acc, lds);
    if (threadIdx.x == 0) {
        if (F.template inside<4>(p.out)) F.template st<float>(p.out, (float)total);
        else F.fault();
    }
}

// ---- RMSNorm -------------------------------------------------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// Nearest bfloat16, ties to even.
__device__ __forceinline__ uint32_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;          // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    return f32_to_bf16(lo) | (f32_to_bf16(hi) << 16);
}

// 512 threads per row (measured against 128, 256 and 1024: 5.5, 5.8 and 5.1 TB/s
// against 6.05 at the bench shape): two 16-byte chunks per thread cover 8192 columns.
// The output is written with nontemporal stores: it is not read again, and with plain stores it
// displaces the input from the caches (4096 x 8192: 6.25 -> 6.6 TB/s, 16384 x 8192: 5.95 -> 7.2,
// 32768 x 4096: 5.55 -> 6.5; nontemporal loads as well as stores are slower than either alone).
// A kernel that keeps several rows per workgroup in flight (gains held in registers, rows copied
// global -> LDS two ahead) was built and measured as well: no faster than this one at any shape.
constexpr int RMS_WG = 512;
// CH: 16-byte chunks (8 values) per thread held in registers -- 2 cover 8192 columns, 4 cover 16384 (the launcher
// picks the smaller that fits: the wider kernel needs twice the registers for the row and the gains)

// Address checking (Sections 4.3, 4.4): the logical thread of y[r,j] reads all of row r,
// then g[j], then stores, and returns at its first refused access.  A row of x that is
// not wholly inside the partition therefore stops -- and counts -- all `cols` threads of
// the row; a refused g[j] or y[r,j] stops that one thread.
// TILE: the launcher has found that the fence maps x, g and y each to one contiguous range (Fence::whole_run on the
// whole matrices; under address checking: all three inside, so that no thread can be refused), the pointers
// 16-byte aligned and the row at most 8192 columns, a multiple of 8.  That instance holds the per-array path alone
// (it repeats the test per row): with every path in one kernel a workgroup ran ~100 scalar instructions and ten
// branches before its first load, which rows of 4096 columns and fewer do not hide (fenced 9-13 % behind
// unfenced there).  The other instance holds the per-lane paths.
template <int V, int CH = 2, bool TILE = false>
__global__ __launch_bounds__(RMS_WG) void k_rmsnorm_bf16(gd_args_rmsnorm p, FenceArgs fa)
{
    const Fence<V> F(fa);
    __shared__ float lds[RMS_WG / 64];
    const uint64_t row = blockIdx.x;
    const uint64_t xrow = p.x + 2 * row * p.cols;
    const uint64_t yrow = p.y + 2 * row * p.cols;
    const float inv_cols = 1.0f / (float)p.cols;
    const bool vec = ((p.x | p.y | p.g) & 15) == 0 && (p.cols & 7) == 0 &&
                     p.cols <= (uint32_t)(RMS_WG * 8 * CH);
    const uint64_t row_bytes = 2 * (uint64_t)p.cols;

    if constexpr (TILE) {
        // (the per-array form only with two chunks: its loads are waited for by hand, and with four conditional loads
        // in flight the compiler moves their registers before the wait -- the ISA audit reports it; the wider kernel
        // fences per lane, with loads the compiler counts)
        static_assert(CH == 2, "the per-array path holds two chunks per thread");
        if (!(vec && F.whole_run(xrow, row_bytes) && F.whole_run(p.g, row_bytes) && F.whole_run(yrow, row_bytes)))
            return;                                                 // never taken: the launcher tested the same for all rows
        // The row, the gains and the output row are each mapped to one contiguous range by the
        // fence (always, unless a pointer wraps at the partition end inside them): their first
        // bytes are fenced once, on the scalar unit, and every wavefront covers 1 KiB tiles at
        // "fenced start + offset".
        const uint32_t chunks = p.cols >> 3;
        const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        const uint32_t lane16 = Fence<V>::template tile_lane_offset<1024>(16 * threadIdx.x);
        const uint64_t fx = F.scalar_fence(xrow), fg = F.scalar_fence(p.g), fy = F.scalar_fence(yrow);
        u32x4 xv[CH], gv[CH];
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const uint32_t q0 = 64 * wave + c * RMS_WG;              // the wavefront's first chunk of this pass over the row
            if (threadIdx.x + c * RMS_WG < chunks) {
                xv[c] = F.template ld_tile16<u32x4>(fx + 16 * (uint64_t)q0, lane16);
                gv[c] = F.template ld_tile16<u32x4>(fg + 16 * (uint64_t)q0, lane16);
            }
        }
        F.tile_wait(xv[0], xv[1]);
        F.tile_wait(gv[0], gv[1]);
        float ss = 0.0f;
#pragma unroll
        for (int c = 0; c < CH; ++c)
            if (threadIdx.x + c * RMS_WG < chunks) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float a = bf16_lo(xv[c][e]), b = bf16_hi(xv[c][e]);
                    ss += a * a;
                    ss += b * b;
                }
            }
        ss = block_sum<RMS_WG / 64>(ss, lds);
        const float inv = 1.0f / sqrtf(ss * inv_cols + p.eps);
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const uint32_t q0 = 64 * wave + c * RMS_WG;
            if (threadIdx.x + c * RMS_WG < chunks) {
                u32x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    o[e] = pack_bf16(bf16_lo(xv[c][e]) * inv * bf16_lo(gv[c][e]),
                                     bf16_hi(xv[c][e]) * inv * bf16_hi(gv[c][e]));
                F.template st_tile16<u32x4, true>(fy + 16 * (uint64_t)q0, lane16, o);
            }
        }
        return;
    }

    if (F.CHECKED && !F.inside_run(xrow, 2 * (uint64_t)p.cols)) {       // workgroup-uniform
        if (threadIdx.x == 0) F.fault(p.cols);
        return;
    }
    // one output element under address checking: false = its thread stops (counted by the caller)
    auto put = [&](uint32_t j, float x, float inv) -> bool {
        if (!F.template inside<2>(p.g + 2 * (uint64_t)j)) return false;
        const float g = bf16_lo(F.template ld<uint16_t>(p.g + 2 * (uint64_t)j));
        if (!F.template inside<2>(yrow + 2 * (uint64_t)j)) return false;
        F.template st<uint16_t>(yrow + 2 * (uint64_t)j, (uint16_t)f32_to_bf16(x * inv * g));
        return true;
    };

    if (vec) {
        const uint32_t chunks = p.cols >> 3;
        u32x4 xv[CH];
        float ss = 0.0f;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const uint32_t q = threadIdx.x + c * RMS_WG;
            if (q < chunks) {
                xv[c] = F.template ld<u32x4>(xrow + 16 * (uint64_t)q);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float a = bf16_lo(xv[c][e]), b = bf16_hi(xv[c][e]);
                    ss += a * a;
                    ss += b * b;
                }
            }
        }
        // the gains do not depend on the row's sum: fetch them before the reduction's barriers
        u32x4 gv[CH];
        bool whole[CH];          // address checking: gain and output chunk both wholly inside
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const uint32_t q = threadIdx.x + c * RMS_WG;
            whole[c] = F.template inside<16>(p.g + 16 * (uint64_t)q) && F.template inside<16>(yrow + 16 * (uint64_t)q);
            if (q < chunks && whole[c]) gv[c] = F.template ld<u32x4>(p.g + 16 * (uint64_t)q);
        }
        ss = block_sum<RMS_WG / 64>(ss, lds);
        const float inv = 1.0f / sqrtf(ss * inv_cols + p.eps);
        uint32_t stopped = 0;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const uint32_t q = threadIdx.x + c * RMS_WG;
            if (q >= chunks) continue;
            if (whole[c]) {
                u32x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    o[e] = pack_bf16(bf16_lo(xv[c][e]) * inv * bf16_lo(gv[c][e]),
                                     bf16_hi(xv[c][e]) * inv * bf16_hi(gv[c][e]));
                F.template st<u32x4, true>(yrow + 16 * (uint64_t)q, o);
            } else {
                for (int e = 0; e < 8; ++e) {
                    const uint32_t w = xv[c][e >> 1];
                    stopped += !put(8 * q + e, (e & 1) ? bf16_hi(w) : bf16_lo(w), inv);
                }
            }
        }
        if (F.CHECKED && stopped) F.fault(stopped);
    } else if (((p.x | p.y | p.g) & 15) == 0 && (p.cols & 7) == 0) {
        // a row wider than the registers hold: read once for the sum and once more, from the caches, for the output
        const uint32_t chunks = p.cols >> 3;
        float ss = 0.0f;
        for (uint32_t q = threadIdx.x; q < chunks; q += RMS_WG) {
            const u32x4 xv = F.template ld<u32x4>(xrow + 16 * (uint64_t)q);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float a = bf16_lo(xv[e]), b = bf16_hi(xv[e]);
                ss += a * a;
                ss += b * b;
            }
        }
        ss = block_sum<RMS_WG / 64>(ss, lds);
        const float inv = 1.0f / sqrtf(ss * inv_cols + p.eps);
        uint32_t stopped = 0;
        for (uint32_t q = threadIdx.x; q < chunks; q += RMS_WG) {
            const u32x4 xv = F.template ld<u32x4>(xrow + 16 * (uint64_t)q);
            if (F.template inside<16>(p.g + 16 * (uint64_t)q) && F.template inside<16>(yrow + 16 * (uint64_t)q)) {
                const u32x4 gv = F.template ld<u32x4>(p.g + 16 * (uint64_t)q);
                u32x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    o[e] = pack_bf16(bf16_lo(xv[e]) * inv * bf16_lo(gv[e]), bf16_hi(xv[e]) * inv * bf16_hi(gv[e]));
                F.template st<u32x4, true>(yrow + 16 * (uint64_t)q, o);
            } else {
                for (int e = 0; e < 8; ++e) {
                    const uint32_t w = xv[e >> 1];
                    stopped += !put(8 * q + e, (e & 1) ? bf16_hi(w) : bf16_lo(w), inv);
                }
            }
        }
        if (F.CHECKED && stopped) F.fault(stopped);
    } else {
        float ss = 0.0f;
        for (uint32_t j = threadIdx.x; j < p.cols; j += RMS_WG) {
            const float a = bf16_lo(F.template ld<uint16_t>(xrow + 2 * (uint64_t)j));
            ss += a * a;
        }
        ss = block_sum<RMS_WG / 64>(ss, lds);
        const float inv = 1.0f / sqrtf(ss * inv_cols + p.eps);
        uint32_t stopped = 0;
        for (uint32_t j = threadIdx.x; j < p.cols; j += RMS_WG)
            stopped += !put(j, bf16_lo(F.template ld<uint16_t>(xrow + 2 * (uint64_t)j)), inv);
        if (F.CHECKED && stopped) F.fault(stopped);
    }
}

// ---- launchers -------------------------------------------------------------------------

constexpr uint32_t SUM_MAX_BLOCKS = 2048;
static_assert(SUM_MAX_BLOCKS * 4 <= GD_SUM_WORKSPACE, "workspace too small for the partial sums");
static_assert(SUM_MAX_BLOCKS <= FIN_WG * FIN_PER, "the second pass reads every partial once");

static uint32_t sum_blocks(uint64_t n)
{
    const uint64_t tile = (uint64_t)WG * SUM_UNROLL * 4;                 // elements per tile
    uint64_t blocks = (n + tile - 1) / tile;
    if (blocks == 0) blocks = 1;
    return (uint32_t)(blocks > SUM_MAX_BLOCKS ? SUM_MAX_BLOCKS : blocks);
}

template <bool OWN_WS>
static int launch_sum(const gd_args_sum &p, const FenceArgs &f, int variant, hipStream_t stream)
{
    const uint32_t blocks = sum_blocks(p.n);
    int rc = with_variant(variant, [&](auto v) {
        hipLaunchKernelGGL((k_sum_partial<decltype(v)::value, OWN_WS>), dim3(blocks), dim3(WG), 0, stream, p, f);
    });
    if (rc != GD_OK) return rc;
    GD_CHECK_LAUNCH();
    rc = with_variant(variant, [&](auto v) {
        hipLaunchKernelGGL((k_sum_final<decltype(v)::value, OWN_WS>), dim3(1), dim3(FIN_WG), 0, stream, p, blocks, f);
    });
    if (rc != GD_OK) return rc;
    GD_CHECK_LAUNCH();
    return GD_OK;
}

int launch_sum_f32(const void *args, const FenceArgs &f, int variant, const Shape &shape, hipStream_t stream)
{
    if (shape.grid || shape.block) return GD_EINVAL;
    return launch_sum<false>(*(const gd_args_sum *)args, f, variant, stream);
}

// ---- the sum without a workspace argument ---------------------------------------------
// The partial sums live in this file-scope device array.  Every GPU the library runs on
// holds its own copy at its own address; in host code the array's name is only a handle
// for hipGetSymbolAddress, never an address to pass to a kernel.  The address is looked
// up once per device, with that device current, and kept.  Nothing in the array has to
// start at zero: pass 1 writes partials[0 .. blocks) before pass 2 reads exactly those.
static_assert(SUM_MAX_BLOCKS * 4 == GD_SUM_NOALLOC_SCRATCH, "header and kernel disagree on the scratch size");
static __device__ __align__(256) float scratch[SUM_MAX_BLOCKS];

constexpr int MAX_DEVICES = 64;
static std::mutex g_scratch_mu;
static void *g_scratch_ptr[MAX_DEVICES];      // device address of `scratch` per device, null = not looked up yet

int launch_sum_f32_noalloc(uint64_t out, uint64_t in, uint64_t n, const FenceArgs &f, int variant,
                           hipStream_t stream)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= MAX_DEVICES) {
        note_hip_error(e != hipSuccess ? e : hipErrorInvalidDevice);
        return GD_EHIP;
    }
    void *ws;
    {
        std::lock_guard<std::mutex> g(g_scratch_mu);
        if (!g_scratch_ptr[dev]) {
            void *ptr = nullptr;
            e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !ptr) {
                note_hip_error(e != hipSuccess ? e : hipErrorInvalidSymbol);
                return GD_EHIP;
            }
            g_scratch_ptr[dev] = ptr;
        }
        ws = g_scratch_ptr[dev];
    }
    const gd_args_sum p = {out, in, (uint64_t)(uintptr_t)ws, n};
    return launch_sum<true>(p, f, variant, stream);
}

int launch_rmsnorm_bf16(const void *args, const FenceArgs &f, int variant, const Shape &shape,
                        hipStream_t stream)
{
    const gd_args_rmsnorm &p = *(const gd_args_rmsnorm *)args;
    if (shape.grid || shape.block) return GD_EINVAL;
    if (p.cols == 0 || p.rows > 0x7fffffffu) return GD_ESHAPE;
    if (p.rows == 0) return GD_OK;
    const bool four = p.cols > (uint32_t)(RMS_WG * 8 * 2);          // beyond 16384 columns either kernel reads the row twice
    const uint64_t row_bytes = 2 * (uint64_t)p.cols;
    const bool tile = !four && (p.cols & 7) == 0 && ((p.x | p.y | p.g) & 15) == 0 &&
                      whole_run_host(f, variant, p.x, row_bytes * p.rows) && whole_run_host(f, variant, p.g, row_bytes) &&
                      whole_run_host(f, variant, p.y, row_bytes * p.rows);
    const int rc = with_variant(variant, [&](auto v) {
        constexpr int V = decltype(v)::value;
        if (four) hipLaunchKernelGGL((k_rmsnorm_bf16<V, 4, false>), dim3(p.rows), dim3(RMS_WG), 0, stream, p, f);
        else if (tile) hipLaunchKernelGGL((k_rmsnorm_bf16<V, 2, true>), dim3(p.rows), dim3(RMS_WG), 0, stream, p, f);
        else hipLaunchKernelGGL((k_rmsnorm_bf16<V, 2, false>), dim3(p.rows), dim3(RMS_WG), 0, stream, p, f);
    });
    if (rc != GD_OK) return rc;
    GD_CHECK_LAUNCH();
    return GD_OK;
}

}  // namespace gd
