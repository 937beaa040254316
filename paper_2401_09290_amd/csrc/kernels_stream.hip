// Contiguous element-wise kernels: Listing 1's sample store, the fence probe,
// STREAM copy and STREAM triad.  HBM-bound: 16 bytes per lane per access with
// the nontemporal hint, one vector per lane and loop trip (measured best: a
// single-wavefront workgroup per 1 KiB tile).  The fence (fence.hpp) is applied to
// the final address of every access; kernels are identical for every variant apart
// from it.
#include <chrono>

#include "launchers.hpp"

namespace gd {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Default workgroup of copy and triad: one wavefront, i.e. one 1 KiB tile per stream and
// workgroup.  Measured against 128..1024 threads: +3 % for a kernel alone, +7 % for eight
// tenants' kernels sharing the chip (the dispatcher interleaves them at a finer grain).
constexpr uint32_t STREAM_BLOCK = 64;

// ---- store_tid: A[i] = j (paper Listing 1 / Section 4.3) -----------------------
template <int V>
__global__ __launch_bounds__(1024) void k_store_tid(gd_args_store_tid p, FenceArgs fa)
{
    const Fence<V> F(fa);
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < p.n; i += stride) {
        const uint64_t a = p.A + 4 * i;
        if (!F.template inside<4>(a)) { F.fault(); continue; }
        F.template st<uint32_t>(a, p.j);
    }
}

// ---- fence probe: out[i] = fence_width(in[i]) ----------------------------------
// Under address checking the probe reports ~0 for an address that is refused (and
// counts it), like any other refused access.
template <int V>
__global__ __launch_bounds__(1024) void k_fence_addrs(gd_args_fence_addrs p, FenceArgs fa)
{
    const Fence<V> F(fa);
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < p.n; i += stride) {
        if (!F.template inside<8>(p.in + 8 * i)) { F.fault(); continue; }
        const uint64_t a = F.template ld<uint64_t>(p.in + 8 * i);
        uint64_t f;
        bool ok;
        switch (p.width) {
        case 1: f = F.template lane_address<1>(a); ok = F.template inside<1>(a); break;
        case 2: f = F.template lane_address<2>(a); ok = F.template inside<2>(a); break;
        case 4: f = F.template lane_address<4>(a); ok = F.template inside<4>(a); break;
        case 8: f = F.template lane_address<8>(a); ok = F.template inside<8>(a); break;
        default: f = F.template lane_address<16>(a); ok = F.template inside<16>(a); break;
        }
        if (!ok) { F.fault(); f = ~(uint64_t)0; }
        if (!F.template inside<8>(p.out + 8 * i)) { F.fault(); continue; }
        F.template st<uint64_t>(p.out + 8 * i, f);
    }
}

// ---- pointer chase: the latency of one fenced access (Section 4.4's model, Figure 5) ----
// Every load depends on the one before it and goes through the per-lane fence, so the time per step is the
// latency of the access plus what the rule adds to the dependent chain.  The first index passes through a vector
// register the compiler knows nothing about: the chain stays on the vector memory path also for one thread.
template <int V>
__global__ __launch_bounds__(64) void k_chase(gd_args_chase p, FenceArgs fa)
{
    const Fence<V> F(fa);
    const uint32_t t = threadIdx.x;
    if (t >= p.threads) return;
    uint32_t idx;
    {
        const uint32_t first = p.start + t * p.lane_step;
        asm volatile("v_mov_b32 %0, %1" : "=v"(idx) : "v"(first));
    }
    const uint64_t cycles0 = __builtin_readcyclecounter();
    const uint64_t ticks0 = __builtin_amdgcn_s_memrealtime();
    for (uint64_t s = 0; s < p.steps; ++s) {
        const uint64_t a = p.tab + 4 * (uint64_t)idx;
        if (!F.template inside<4>(a)) { F.fault(); return; }
        idx = F.template ld<uint32_t>(a);
    }
    asm volatile("" : "+v"(idx));                        // the last load has landed before the clocks are read again
    const uint64_t cycles = __builtin_readcyclecounter() - cycles0;
    const uint64_t ticks = __builtin_amdgcn_s_memrealtime() - ticks0;
    if (!F.template inside<4>(p.out + 4 * (uint64_t)t)) { F.fault(); return; }
    F.template st<uint32_t>(p.out + 4 * (uint64_t)t, idx);
    if (t != 0) return;
    if (!F.template inside<8>(p.clk)) { F.fault(); return; }
    F.template st<uint64_t>(p.clk, cycles);
    if (!F.template inside<8>(p.clk + 8)) { F.fault(); return; }
    F.template st<uint64_t>(p.clk + 8, ticks);
}

// ---- copy / triad ------------------------------------------------------------------
// OP 0: a = b.  OP 1: a = b + s*c (one fused multiply-add per element).
// Vector path when all pointers are 16-byte aligned (then a 16-byte access equals
// four fenced 4-byte accesses); otherwise every element is accessed on its own.
// On the vector path a wavefront covers one contiguous 1 KiB tile of each array.  If the
// fence maps each array to one contiguous range (Fence::whole_run, tested once per launch:
// always, unless a pointer wraps at the partition end inside its array) each array's first
// byte is fenced once, on the scalar unit, and the loop addresses "fenced start + offset"
// with the instructions of the native kernel; otherwise every vector is fenced per lane.
// Under address checking a vector whose three 16-byte accesses are not all inside
// the partition is redone element by element, so that exactly the offending
// logical threads stop.
constexpr int STREAM_TILE = 1024;      // bytes per wavefront and array: 64 lanes x 16 bytes

// NT: the vector accesses carry the nontemporal hint (data touched once).  A launch that
// repeats its pass keeps the hint off, so that the caches may hold its working set.
template <int V, int OP, bool NT>
__global__ __launch_bounds__(1024) void k_stream(uint64_t pa, uint64_t pb, uint64_t pc, uint64_t n,
                                                 float s, uint32_t repeat, FenceArgs fa)
{
    const Fence<V> F(fa);
    // Launch-invariant: are all pointers 16-byte aligned, does the fence map each array to one
    // contiguous range, and where does each array's first byte go.
    const uint64_t ptr_bits = OP ? (pa | pb | pc) : (pa | pb);
    const uint64_t n4 = n >> 2;
    const bool whole = F.whole_run(pb, 16 * n4) && (!OP || F.whole_run(pc, 16 * n4)) && F.whole_run(pa, 16 * n4);
    const uint64_t fb = F.scalar_fence(pb), fc = OP ? F.scalar_fence(pc) : 0, fa_ = F.scalar_fence(pa);   // used only if `whole`
    // one logical thread: accesses in the order load b, load c, store a
    auto element = [&](uint64_t i) {
        if (!F.template inside<4>(pb + 4 * i)) { F.fault(); return; }
        float r = F.template ld<float>(pb + 4 * i);
        if (OP) {
            if (!F.template inside<4>(pc + 4 * i)) { F.fault(); return; }
            r = r + s * F.template ld<float>(pc + 4 * i);
        }
        if (!F.template inside<4>(pa + 4 * i)) { F.fault(); return; }
        F.template st<float>(pa + 4 * i, r);
    };
    auto tail = [&]() {                                   // at most three elements behind the last whole vector
        if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {
            uint64_t i = 4 * n4 + threadIdx.x;
            asm volatile("" : "+v"(i));                   // nothing of this is hoisted in front of the vectors
            element(i);
        }
    };
    const bool aligned = (ptr_bits & 15) == 0;
    const uint64_t step = (uint64_t)gridDim.x * blockDim.x;
    // repeat > 1 runs the pass again (the cache-resident regime in one launch); the loop over the passes sits inside
    // the choice of the path, so that a pass jumps over no code of the paths it does not take
    if (aligned && whole) {
        // every array is mapped to one contiguous range and its first byte is fenced: address it like a native kernel
        const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        const uint32_t lane_off = Fence<V>::template tile_lane_offset<STREAM_TILE>(16 * threadIdx.x);
        for (uint32_t rep = 0; rep < repeat; ++rep) {
            for (uint64_t w0 = (uint64_t)blockIdx.x * blockDim.x + 64 * wave; w0 < n4; w0 += step) {   // w0: the tile's first vector
                if (w0 + (threadIdx.x & 63) >= n4) continue;
                f32x4 vb = F.template ld_tile16<f32x4, NT>(fb + 16 * w0, lane_off);
                if (OP) {
                    f32x4 vc = F.template ld_tile16<f32x4, NT>(fc + 16 * w0, lane_off);
                    F.tile_wait(vb, vc);
                    vb = vb + s * vc;
                } else {
                    F.tile_wait(vb);
                }
                // the copy also writes through at device scope (+1 to 2 % from 2^26 elements up); the triad gains nothing
                // from that at 2^27 and 2^28 and loses 1.5 to 7 % at 2^24 to 2^26
                F.template st_tile16<f32x4, NT, OP == 0>(fa_ + 16 * w0, lane_off, vb);
            }
            tail();
        }
    } else if (aligned) {
        // a pointer wraps at the partition end inside its array (or, under address checking, an array is
        // not wholly inside): every vector is fenced (checked) per lane
        for (uint32_t rep = 0; rep < repeat; ++rep) {
            for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += step) {
                if (F.CHECKED &&
                    !(F.template inside<16>(pb + 16 * i) && (!OP || F.template inside<16>(pc + 16 * i)) &&
                      F.template inside<16>(pa + 16 * i))) {
                    for (int e = 0; e < 4; ++e) element(4 * i + e);
                } else {
                    f32x4 v = F.template ld<f32x4, NT>(pb + 16 * i);
                    if (OP) v = v + s * F.template ld<f32x4, NT>(pc + 16 * i);
                    F.template st<f32x4, NT>(pa + 16 * i, v);
                }
            }
            tail();
        }
    } else {
        for (uint32_t rep = 0; rep < repeat; ++rep)
            for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += step) element(i);
    }
}

// ---- launchers -------------------------------------------------------------------

int launch_store_tid(const void *args, const FenceArgs &f, int variant, const Shape &shape,
                     hipStream_t stream)
{
    const gd_args_store_tid &p = *(const gd_args_store_tid *)args;
    uint32_t grid, block;
    if (!pick_1d(shape, (p.n + 255) / 256, 256, &grid, &block)) return GD_EINVAL;
    if (p.n == 0) return GD_OK;
    const int rc = with_variant(variant, [&](auto v) {
        hipLaunchKernelGGL((k_store_tid<decltype(v)::value>), dim3(grid), dim3(block), 0, stream, p, f);
    });
    if (rc != GD_OK) return rc;
    GD_CHECK_LAUNCH();
    return GD_OK;
}

int probe_raw_launches(const gd_args_store_tid &p, const FenceArgs &f, int variant, uint32_t iters, hipStream_t stream,
                       double *ns_per_call)
{
    void (*kernel)(gd_args_store_tid, FenceArgs) = nullptr;
    const int rc = with_variant(variant, [&](auto v) { kernel = k_store_tid<decltype(v)::value>; });
    if (rc != GD_OK) return rc;
    const auto t0 = std::chrono::steady_clock::now();
    for (uint32_t i = 0; i < iters; ++i) hipLaunchKernelGGL(kernel, dim3(1), dim3(256), 0, stream, p, f);   // the shape launch_store_tid picks for 64 elements
    const auto t1 = std::chrono::steady_clock::now();
    GD_CHECK_LAUNCH();
    *ns_per_call = std::chrono::duration<double, std::nano>(t1 - t0).count() / iters;
    return GD_OK;
}

int launch_chase(const void *args, const FenceArgs &f, int variant, const Shape &shape, hipStream_t stream)
{
    const gd_args_chase &p = *(const gd_args_chase *)args;
    if (shape.grid || shape.block) return GD_EINVAL;
    if (p.threads == 0 || p.threads > 64) return GD_ESHAPE;
    const int rc = with_variant(variant, [&](auto v) {
        hipLaunchKernelGGL((k_chase<decltype(v)::value>), dim3(1), dim3(64), 0, stream, p, f);
    });
    if (rc != GD_OK) return rc;
    GD_CHECK_LAUNCH();
    return GD_OK;
}

int launch_fence_addrs(const void *args, const FenceArgs &f, int variant, const Shape &shape,
                       hipStream_t stream)
{
    const gd_args_fence_addrs &p = *(const gd_args_fence_addrs *)args;
    if (!(p.width == 1 || p.width == 2 || p.width == 4 || p.width == 8 || p.width == 16))
        return GD_ESHAPE;
    uint32_t grid, block;
    if (!pick_1d(shape, (p.n + 255) / 256, 256, &grid, &block)) return GD_EINVAL;
    if (p.n == 0) return GD_OK;
    const int rc = with_variant(variant, [&](auto v) {
        hipLaunchKernelGGL((k_fence_addrs<decltype(v)::value>), dim3(grid), dim3(block), 0, stream, p, f);
    });
    if (rc != GD_OK) return rc;
    GD_CHECK_LAUNCH();
    return GD_OK;
}

static uint64_t stream_tiles(uint64_t n, uint32_t block) { return ((n >> 2) + block - 1) / block; }

template <int OP>
static int launch_stream(uint64_t a, uint64_t b, uint64_t c, uint64_t n, float s, uint32_t repeat,
                         const FenceArgs &f, int variant, const Shape &shape, hipStream_t stream)
{
    const uint32_t b0 = shape.block ? shape.block[0] : STREAM_BLOCK;
    uint32_t grid, block;
    if (!pick_1d(shape, b0 ? stream_tiles(n, b0) : 1, STREAM_BLOCK, &grid, &block)) return GD_EINVAL;
    if (n == 0) return GD_OK;
    const int rc = with_variant(variant, [&](auto v) {
        constexpr int V = decltype(v)::value;
        if (repeat > 1) hipLaunchKernelGGL((k_stream<V, OP, false>), dim3(grid), dim3(block), 0, stream, a, b, c, n, s, repeat, f);
        else hipLaunchKernelGGL((k_stream<V, OP, true>), dim3(grid), dim3(block), 0, stream, a, b, c, n, s, 1u, f);
    });
    if (rc != GD_OK) return rc;
    GD_CHECK_LAUNCH();
    return GD_OK;
}

int launch_copy(const void *args, const FenceArgs &f, int variant, const Shape &shape, hipStream_t stream)
{
    const gd_args_copy &p = *(const gd_args_copy *)args;
    return launch_stream<0>(p.a, p.b, 0, p.n, 0.0f, 1, f, variant, shape, stream);
}

int launch_triad(const void *args, const FenceArgs &f, int variant, const Shape &shape, hipStream_t stream)
{
    const gd_args_triad &p = *(const gd_args_triad *)args;
    return launch_stream<1>(p.a, p.b, p.c, p.n, p.s, p.repeat, f, variant, shape, stream);
}

}  // namespace gd
