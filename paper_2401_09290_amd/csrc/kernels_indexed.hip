// Indexed kernels: saxpy through int32 element offsets, gather and scatter of
// 4-byte values through int64 or int32 indices.  The index/offset stream and the
// contiguous side are read or written 16 bytes per lane; the data-dependent side
// is one 4-byte access per element, each with the fence on its final address
// (index * 4 added to the tenant's pointer in wrap-around arithmetic, then
// fenced -- the register+offset rule of Section 4.3).
#include "launchers.hpp"

namespace gd {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
typedef uint64_t u64x2 __attribute__((ext_vector_type(2)));

constexpr int EPT = 4;   // elements per thread on the vector path

// Under address checking (Section 4.4) the kernels take their per-element path,
// where every access is tested on its own and an offending logical thread stops.
//
// The contiguous streams of the vector path (indices, offsets, the gather's output, the
// scatter's source) are covered by each wavefront in tiles of 1 KiB (16 bytes per lane) or
// 2 KiB (32 bytes per lane, as two 16-byte halves).  If the fence maps each of these arrays
// to one contiguous range (Fence::whole_run: always, unless a pointer wraps at the partition
// end) the kernel fences each stream's first byte once, on the scalar unit, and runs its
// tile loop, which addresses the streams as "fenced start + offset" like a native kernel;
// only the data-dependent accesses are fenced per lane.

// ---- y[o] = alpha*x[o] + y[o], o = off[i] ---------------------------------------
template <int V>
__global__ __launch_bounds__(1024) void k_saxpy_idx(gd_args_saxpy_idx p, FenceArgs fa)
{
    const Fence<V> F(fa);
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    const uint64_t tid = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint64_t done = 0;
    if (!F.CHECKED && (p.off & 15) == 0) {
        const uint64_t n4 = p.n >> 2;
        // all eight fenced addresses first, in registers of their own (Fence::keep_apart), then the loads, then the stores
        auto four = [&](const i32x4 o) {
            typename Fence<V>::Handle hx[EPT], hy[EPT];
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                const uint64_t byte_off = (uint64_t)((int64_t)o[e] * 4);
                hx[e] = F.template fenced<4>(p.x + byte_off);
                hy[e] = F.template fenced<4>(p.y + byte_off);
            }
            Fence<V>::keep_apart(hx[0], hx[1], hx[2], hx[3]);
            Fence<V>::keep_apart(hy[0], hy[1], hy[2], hy[3]);
            float vx[EPT], vy[EPT];
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                vx[e] = F.template ld_fenced<float>(hx[e]);
                vy[e] = F.template ld_fenced<float>(hy[e]);
            }
#pragma unroll
            for (int e = 0; e < EPT; ++e) F.template st_fenced<float>(hy[e], p.alpha * vx[e] + vy[e]);
        };
        if (F.whole_run(p.off, 16 * n4)) {
            const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
            const uint32_t lane16 = Fence<V>::template tile_lane_offset<1024>(16 * threadIdx.x);
            const uint64_t f_off = F.scalar_fence(p.off);                      // fenced first byte of the offsets
            // q0: the wavefront's first vector (scalar registers); q: this lane's
            for (uint64_t q0 = (uint64_t)blockIdx.x * blockDim.x + 64 * wave; q0 < n4; q0 += stride) {
                if (q0 + (threadIdx.x & 63) >= n4) continue;
                i32x4 o = F.template ld_tile16<i32x4, true>(f_off + 16 * q0, lane16);
                F.tile_wait(o);
                four(o);
            }
        } else {
            for (uint64_t q = tid; q < n4; q += stride) four(F.template ld<i32x4, true>(p.off + 16 * q));
        }
        done = 4 * n4;
    }
    for (uint64_t i = done + tid; i < p.n; i += stride) {
        if (!F.template inside<4>(p.off + 4 * i)) { F.fault(); continue; }
        const int32_t o = F.template ld<int32_t>(p.off + 4 * i);
        const uint64_t byte_off = (uint64_t)((int64_t)o * 4);
        if (!F.template inside<4>(p.x + byte_off)) { F.fault(); continue; }
        const float vx = F.template ld<float>(p.x + byte_off);
        if (!F.template inside<4>(p.y + byte_off)) { F.fault(); continue; }
        const float vy = F.template ld<float>(p.y + byte_off);
        F.template st<float>(p.y + byte_off, p.alpha * vx + vy);
    }
}

// ---- out[i] = tab[idx[i]] --------------------------------------------------------
// IDX64: 1 = int64 indices, 0 = int32 indices (sign-extended).
template <int V, int IDX64>
__global__ __launch_bounds__(1024) void k_gather32(gd_args_gather p, FenceArgs fa)
{
    const Fence<V> F(fa);
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    const uint64_t tid = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint64_t done = 0;
    if (!F.CHECKED && ((p.idx | p.out) & 15) == 0) {
        const uint64_t n4 = p.n >> 2;
        auto four = [&](const uint64_t (&k)[EPT]) {
            u32x4 v;
#pragma unroll
            for (int e = 0; e < EPT; ++e) v[e] = F.template ld<uint32_t>(p.tab + 4 * k[e]);
            return v;
        };
        if (F.whole_run(p.idx, (IDX64 ? 32 : 16) * n4) && F.whole_run(p.out, 16 * n4)) {
            const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
            const uint32_t lane16 = Fence<V>::template tile_lane_offset<1024>(16 * threadIdx.x);
            const uint32_t lane32 = Fence<V>::template tile_lane_offset<2048>(32 * threadIdx.x);
            const uint64_t f_idx = F.scalar_fence(p.idx), f_out = F.scalar_fence(p.out);   // fenced first bytes of the streams
            // q0: the wavefront's first vector (scalar registers); q: this lane's
            for (uint64_t q0 = (uint64_t)blockIdx.x * blockDim.x + 64 * wave; q0 < n4; q0 += stride) {
                if (q0 + (threadIdx.x & 63) >= n4) continue;
                uint64_t k[EPT];
                if (IDX64) {
                    const uint64_t t_idx = f_idx + 32 * q0;
                    u64x2 k01 = F.template ld_tile16<u64x2, true>(t_idx, lane32);
                    u64x2 k23 = F.template ld_tile16<u64x2, true, 16>(t_idx, lane32);
                    F.tile_wait(k01, k23);
                    k[0] = k01[0]; k[1] = k01[1]; k[2] = k23[0]; k[3] = k23[1];
                } else {
                    i32x4 k4 = F.template ld_tile16<i32x4, true>(f_idx + 16 * q0, lane16);
                    F.tile_wait(k4);
#pragma unroll
                    for (int e = 0; e < EPT; ++e) k[e] = (uint64_t)(int64_t)k4[e];
                }
                F.template st_tile16<u32x4, true>(f_out + 16 * q0, lane16, four(k));
            }
        } else {
            for (uint64_t q = tid; q < n4; q += stride) {
                uint64_t k[EPT];
                if (IDX64) {
                    const u64x2 k01 = F.template ld<u64x2, true>(p.idx + 32 * q);
                    const u64x2 k23 = F.template ld<u64x2, true>(p.idx + 32 * q + 16);
                    k[0] = k01[0]; k[1] = k01[1]; k[2] = k23[0]; k[3] = k23[1];
                } else {
                    const i32x4 k4 = F.template ld<i32x4, true>(p.idx + 16 * q);
#pragma unroll
                    for (int e = 0; e < EPT; ++e) k[e] = (uint64_t)(int64_t)k4[e];
                }
                F.template st<u32x4, true>(p.out + 16 * q, four(k));
            }
        }
        done = 4 * n4;
    }
    for (uint64_t i = done + tid; i < p.n; i += stride) {
        const uint64_t ia = IDX64 ? p.idx + 8 * i : p.idx + 4 * i;
        if (!F.template inside<IDX64 ? 8 : 4>(ia)) { F.fault(); continue; }
        const uint64_t k = IDX64 ? F.template ld<uint64_t>(ia) : (uint64_t)(int64_t)F.template ld<int32_t>(ia);
        if (!F.template inside<4>(p.tab + 4 * k)) { F.fault(); continue; }
        const uint32_t v = F.template ld<uint32_t>(p.tab + 4 * k);
        if (!F.template inside<4>(p.out + 4 * i)) { F.fault(); continue; }
        F.template st<uint32_t>(p.out + 4 * i, v);
    }
}

// ---- dst[idx[i]] = scale * src[i] -------------------------------------------------
template <int V>
__global__ __launch_bounds__(1024) void k_scatter_f32_i64(gd_args_scatter p, FenceArgs fa)
{
    const Fence<V> F(fa);
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    const uint64_t tid = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint64_t done = 0;
    if (!F.CHECKED && ((p.idx | p.src) & 15) == 0) {
        const uint64_t n4 = p.n >> 2;
        // all four fenced addresses and values first, in registers of their own, then the four stores back to back
        using Handle = typename Fence<V>::Handle;
        auto stores = [&](Handle h0, Handle h1, Handle h2, Handle h3, const f32x4 v) {
            float d0 = p.scale * v[0], d1 = p.scale * v[1], d2 = p.scale * v[2], d3 = p.scale * v[3];
            Fence<V>::keep_apart(h0, h1, h2, h3, d0, d1, d2, d3);
            F.template st_fenced<float>(h0, d0);
            F.template st_fenced<float>(h1, d1);
            F.template st_fenced<float>(h2, d2);
            F.template st_fenced<float>(h3, d3);
        };
        auto four = [&](const u64x2 k01, const u64x2 k23, const f32x4 v) {
            stores(F.template fenced<4>(p.dst + 4 * k01[0]), F.template fenced<4>(p.dst + 4 * k01[1]),
                   F.template fenced<4>(p.dst + 4 * k23[0]), F.template fenced<4>(p.dst + 4 * k23[1]), v);
        };
        // measured: the nontemporal hint on the source stream slows the scattered stores
        if (F.whole_run(p.idx, 32 * n4) && F.whole_run(p.src, 16 * n4)) {
            const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
            const uint32_t lane16 = Fence<V>::template tile_lane_offset<1024>(16 * threadIdx.x);
            const uint32_t lane32 = Fence<V>::template tile_lane_offset<2048>(32 * threadIdx.x);
            const uint64_t f_idx = F.scalar_fence(p.idx), f_src = F.scalar_fence(p.src);   // fenced first bytes of the streams
            // q0: the wavefront's first vector (scalar registers); q: this lane's
            for (uint64_t q0 = (uint64_t)blockIdx.x * blockDim.x + 64 * wave; q0 < n4; q0 += stride) {
                if (q0 + (threadIdx.x & 63) >= n4) continue;
                const uint64_t t_idx = f_idx + 32 * q0;
                u64x2 k01 = F.template ld_tile16<u64x2, true>(t_idx, lane32);
                u64x2 k23 = F.template ld_tile16<u64x2, true, 16>(t_idx, lane32);
                f32x4 v = F.template ld_tile16<f32x4>(f_src + 16 * q0, lane16);
                // the indices are back first: their four addresses are fenced while the values are still on the way
                F.tile_wait_all_but_last(k01, k23);
                Handle h0 = F.template fenced<4>(p.dst + 4 * k01[0]), h1 = F.template fenced<4>(p.dst + 4 * k01[1]),
                       h2 = F.template fenced<4>(p.dst + 4 * k23[0]), h3 = F.template fenced<4>(p.dst + 4 * k23[1]);
                Fence<V>::keep_apart(h0, h1, h2, h3);
                F.tile_wait(v);
                stores(h0, h1, h2, h3, v);
            }
        } else {
            for (uint64_t q = tid; q < n4; q += stride)
                four(F.template ld<u64x2, true>(p.idx + 32 * q), F.template ld<u64x2, true>(p.idx + 32 * q + 16),
                     F.template ld<f32x4>(p.src + 16 * q));
        }
        done = 4 * n4;
    }
    for (uint64_t i = done + tid; i < p.n; i += stride) {
        if (!F.template inside<8>(p.idx + 8 * i)) { F.fault(); continue; }
        const uint64_t k = F.template ld<uint64_t>(p.idx + 8 * i);
        if (!F.template inside<4>(p.src + 4 * i)) { F.fault(); continue; }
        const float v = F.template ld<float>(p.src + 4 * i);
        if (!F.template inside<4>(p.dst + 4 * k)) { F.fault(); continue; }
        F.template st<float>(p.dst + 4 * k, p.scale * v);
    }
}

// ---- measurement aid: does a cache-policy bit change what a random 4-byte load costs? ----------
// The gather of k_gather32 with 64-bit indices, unfenced, in bounds only, with the table
// load written out so that it can carry any combination of the sc0 / sc1 / nt bits
// (POLICY bit 0 = sc0, bit 1 = sc1, bit 2 = nt).  Index and output streams as in the
// library kernel.  Used by bench.py to show that the memory system fills a whole
// 128-byte line per random access whatever the bits say.
template <int POLICY>
__device__ __forceinline__ uint32_t ld_with_policy(const uint32_t *base, uint32_t off)
{
    uint32_t v;
    if constexpr (POLICY == 0) asm volatile("global_load_dword %0, %1, %2" : "=v"(v) : "v"(off), "s"(base) : "memory");
    if constexpr (POLICY == 1) asm volatile("global_load_dword %0, %1, %2 sc0" : "=v"(v) : "v"(off), "s"(base) : "memory");
    if constexpr (POLICY == 2) asm volatile("global_load_dword %0, %1, %2 sc1" : "=v"(v) : "v"(off), "s"(base) : "memory");
    if constexpr (POLICY == 3) asm volatile("global_load_dword %0, %1, %2 sc0 sc1" : "=v"(v) : "v"(off), "s"(base) : "memory");
    if constexpr (POLICY == 4) asm volatile("global_load_dword %0, %1, %2 nt" : "=v"(v) : "v"(off), "s"(base) : "memory");
    if constexpr (POLICY == 5) asm volatile("global_load_dword %0, %1, %2 sc0 nt" : "=v"(v) : "v"(off), "s"(base) : "memory");
    if constexpr (POLICY == 6) asm volatile("global_load_dword %0, %1, %2 sc1 nt" : "=v"(v) : "v"(off), "s"(base) : "memory");
    if constexpr (POLICY == 7) asm volatile("global_load_dword %0, %1, %2 sc0 sc1 nt" : "=v"(v) : "v"(off), "s"(base) : "memory");
    return v;
}

template <int POLICY>
__global__ __launch_bounds__(256) void k_probe_gather_policy(uint32_t *out, const uint32_t *tab, const uint64_t *idx, uint64_t n4)
{
    for (uint64_t q = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; q < n4; q += (uint64_t)gridDim.x * blockDim.x) {
        const u64x2 k01 = __builtin_nontemporal_load((const u64x2 *)(idx + 4 * q));
        const u64x2 k23 = __builtin_nontemporal_load((const u64x2 *)(idx + 4 * q + 2));
        u32x4 v;
        v[0] = ld_with_policy<POLICY>(tab, (uint32_t)(4 * k01[0]));
        v[1] = ld_with_policy<POLICY>(tab, (uint32_t)(4 * k01[1]));
        v[2] = ld_with_policy<POLICY>(tab, (uint32_t)(4 * k23[0]));
        v[3] = ld_with_policy<POLICY>(tab, (uint32_t)(4 * k23[1]));
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(v) : : "memory");
        __builtin_nontemporal_store(v, (u32x4 *)(out + 4 * q));
    }
}

// The caller guarantees that every index is below table_elems and that table_elems * 4 fits 32 bits.
int launch_probe_gather_policy(uint64_t out, uint64_t tab, uint64_t idx, uint64_t n, uint32_t policy, hipStream_t stream)
{
    if (!out || !tab || !idx || ((out | idx) & 15) || (tab & 3) || (n & 3) || policy > 7) return GD_EINVAL;
    if (n == 0) return GD_OK;
    const uint64_t n4 = n >> 2;
    const dim3 grid((uint32_t)((n4 + 255) / 256 > 0x7fffffffull ? 0x7fffffffull : (n4 + 255) / 256)), block(256);
    uint32_t *o = (uint32_t *)(uintptr_t)out;
    const uint32_t *t = (const uint32_t *)(uintptr_t)tab;
    const uint64_t *i = (const uint64_t *)(uintptr_t)idx;
    switch (policy) {
    case 0: hipLaunchKernelGGL((k_probe_gather_policy<0>), grid, block, 0, stream, o, t, i, n4); break;
    case 1: hipLaunchKernelGGL((k_probe_gather_policy<1>), grid, block, 0, stream, o, t, i, n4); break;
    case 2: hipLaunchKernelGGL((k_probe_gather_policy<2>), grid, block, 0, stream, o, t, i, n4); break;
    case 3: hipLaunchKernelGGL((k_probe_gather_policy<3>), grid, block, 0, stream, o, t, i, n4); break;
    case 4: hipLaunchKernelGGL((k_probe_gather_policy<4>), grid, block, 0, stream, o, t, i, n4); break;
    case 5: hipLaunchKernelGGL((k_probe_gather_policy<5>), grid, block, 0, stream, o, t, i, n4); break;
    case 6: hipLaunchKernelGGL((k_probe_gather_policy<6>), grid, block, 0, stream, o, t, i, n4); break;
    default: hipLaunchKernelGGL((k_probe_gather_policy<7>), grid, block, 0, stream, o, t, i, n4); break;
    }
    GD_CHECK_LAUNCH();
    return GD_OK;
}

// ---- launchers ---------------------------------------------------------------------

static uint64_t blocks_for(uint64_t n, uint32_t block)
{
    const uint64_t per_block = (uint64_t)block * EPT;
    return (n + per_block - 1) / per_block;
}

// One launcher body for the four kernels: `launch(v, grid, block)` issues the
// instance for fence variant decltype(v)::value.
template <typename ARGS, typename L>
static int launch_indexed(const ARGS &p, int variant, const Shape &shape, L &&launch)
{
    const uint32_t b0 = shape.block ? shape.block[0] : 256;
    uint32_t grid, block;
    if (!pick_1d(shape, b0 ? blocks_for(p.n, b0) : 1, 256, &grid, &block)) return GD_EINVAL;
    if (p.n == 0) return GD_OK;
    const int rc = with_variant(variant, [&](auto v) { launch(v, dim3(grid), dim3(block)); });
    if (rc != GD_OK) return rc;
    GD_CHECK_LAUNCH();
    return GD_OK;
}

int launch_saxpy_idx(const void *args, const FenceArgs &f, int variant, const Shape &shape, hipStream_t stream)
{
    const gd_args_saxpy_idx &p = *(const gd_args_saxpy_idx *)args;
    return launch_indexed(p, variant, shape, [&](auto v, dim3 g, dim3 b) {
        hipLaunchKernelGGL((k_saxpy_idx<decltype(v)::value>), g, b, 0, stream, p, f);
    });
}

int launch_gather32_i64(const void *args, const FenceArgs &f, int variant, const Shape &shape, hipStream_t stream)
{
    const gd_args_gather &p = *(const gd_args_gather *)args;
    return launch_indexed(p, variant, shape, [&](auto v, dim3 g, dim3 b) {
        hipLaunchKernelGGL((k_gather32<decltype(v)::value, 1>), g, b, 0, stream, p, f);
    });
}

int launch_gather32_i32(const void *args, const FenceArgs &f, int variant, const Shape &shape, hipStream_t stream)
{
    const gd_args_gather &p = *(const gd_args_gather *)args;
    return launch_indexed(p, variant, shape, [&](auto v, dim3 g, dim3 b) {
        hipLaunchKernelGGL((k_gather32<decltype(v)::value, 0>), g, b, 0, stream, p, f);
    });
}

int launch_scatter_f32_i64(const void *args, const FenceArgs &f, int variant, const Shape &shape, hipStream_t stream)
{
    const gd_args_scatter &p = *(const gd_args_scatter *)args;
    return launch_indexed(p, variant, shape, [&](auto v, dim3 g, dim3 b) {
        hipLaunchKernelGGL((k_scatter_f32_i64<decltype(v)::value>), g, b, 0, stream, p, f);
    });
}

}  // namespace gd
