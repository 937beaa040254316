// Per-kernel launchers: each validates the shape on the host, picks the launch
// geometry, and launches the template instance for the requested fence variant.
#pragma once

#include <hip/hip_runtime.h>

#include <type_traits>

#include "../../include/guardian.h"
#include "fence.hpp"

namespace gd {

// Launch geometry requested by the caller: grid/block may be null (library default).
struct Shape {
    const uint32_t *grid;
    const uint32_t *block;
};

using Launcher = int (*)(const void *args, const FenceArgs &f, int variant, const Shape &shape,
                         hipStream_t stream);

int launch_store_tid(const void *, const FenceArgs &, int, const Shape &, hipStream_t);
int launch_fence_addrs(const void *, const FenceArgs &, int, const Shape &, hipStream_t);
int launch_chase(const void *, const FenceArgs &, int, const Shape &, hipStream_t);
int launch_copy(const void *, const FenceArgs &, int, const Shape &, hipStream_t);
int launch_triad(const void *, const FenceArgs &, int, const Shape &, hipStream_t);
int launch_saxpy_idx(const void *, const FenceArgs &, int, const Shape &, hipStream_t);
int launch_gather32_i64(const void *, const FenceArgs &, int, const Shape &, hipStream_t);
int launch_scatter_f32_i64(const void *, const FenceArgs &, int, const Shape &, hipStream_t);
int launch_gather32_i32(const void *, const FenceArgs &, int, const Shape &, hipStream_t);
int launch_sum_f32(const void *, const FenceArgs &, int, const Shape &, hipStream_t);
int launch_rmsnorm_bf16(const void *, const FenceArgs &, int, const Shape &, hipStream_t);
int launch_gemm_bf16(const void *, const FenceArgs &, int, const Shape &, hipStream_t);

// The sum with its partial results in a file-scope device array of the library
// instead of a tenant workspace (gd_sum_f32_noalloc).
int launch_sum_f32_noalloc(uint64_t out, uint64_t in, uint64_t n, const FenceArgs &, int variant, hipStream_t);

// Matrix-pipe probe (gd_probe_mfma): no tenant, no fence.
int launch_mfma_probe(uint64_t operands, uint64_t out, uint32_t blocks, uint32_t iters, hipStream_t);

// Host-path probe (gd_probe_host_path): `iters` bare HIP launches of the store_tid kernel built for
// `variant`, arguments prepared once; *ns_per_call = mean host time of the launch call.
int probe_raw_launches(const gd_args_store_tid &p, const FenceArgs &f, int variant, uint32_t iters, hipStream_t,
                       double *ns_per_call);

// Cache-policy probe of random 4-byte loads (gd_probe_gather_policy): no tenant, no fence.
int launch_probe_gather_policy(uint64_t out, uint64_t tab, uint64_t idx, uint64_t n, uint32_t policy, hipStream_t);

// 1-D launch shape of an element-wise kernel that loops over `tiles` tiles.
// Returns false if the caller's shape is unusable.
inline bool pick_1d(const Shape &s, uint64_t tiles, uint32_t default_block, uint32_t *grid,
                    uint32_t *block)
{
    uint32_t b = default_block;
    uint64_t g = tiles ? tiles : 1;
    if (s.block) {
        b = s.block[0];
        if (b == 0 || b > 1024 || (b % 64) != 0 || s.block[1] > 1 || s.block[2] > 1) return false;
    }
    if (s.grid) {
        if (s.grid[0] == 0 || s.grid[1] > 1 || s.grid[2] > 1) return false;
        g = s.grid[0];
    }
    if (g > 0x7fffffffull) g = 0x7fffffffull;
    *grid = (uint32_t)g;
    *block = b;
    return true;
}

// The one switch from the fence variant chosen on the host to a template instance:
// calls launch(std::integral_constant<int, V>{}), e.g.
//     with_variant(variant, [&](auto v) { hipLaunchKernelGGL((k<decltype(v)::value>), ...); });
template <typename F>
inline int with_variant(int variant, F &&launch)
{
    switch (variant) {
    case V_NONE:  launch(std::integral_constant<int, V_NONE>{});  return GD_OK;
    case V_BIT32: launch(std::integral_constant<int, V_BIT32>{}); return GD_OK;
    case V_BIT64: launch(std::integral_constant<int, V_BIT64>{}); return GD_OK;
    case V_MOD:   launch(std::integral_constant<int, V_MOD>{});   return GD_OK;
    case V_CHECK: launch(std::integral_constant<int, V_CHECK>{}); return GD_OK;
    case V_BUF:   launch(std::integral_constant<int, V_BUF>{});   return GD_OK;
    default: return GD_ENOKERNEL;
    }
}

// Host twin of Fence<V>::whole_run: the fence maps [start, start + bytes) to one contiguous range (under
// address checking: the range lies inside the partition).  Launchers use it to choose a kernel that fences an
// array once; such a kernel repeats the test on the device.
inline bool whole_run_host(const FenceArgs &f, int variant, uint64_t start, uint64_t bytes)
{
    if (variant == V_NONE || variant == V_BUF) return true;
    if (variant == V_BIT32 || variant == V_BIT64) return (((start & f.mask) + (bytes ? bytes - 1 : 0)) & ~f.mask) == 0;
    const uint64_t size = f.mask;
    if (bytes > size) return false;
    const uint64_t diff = start - f.base;                       // wrap-around, as on the device
    if (variant == V_CHECK) return diff <= size - bytes;
    return diff % size <= size - bytes;                          // V_MOD: the image of the first byte has `bytes` bytes behind it
}

// Last HIP error seen by a launcher on this thread (0 = hipSuccess).
void note_hip_error(hipError_t e);
#define GD_CHECK_LAUNCH()                                  \
    do {                                                   \
        hipError_t e_ = hipGetLastError();                 \
        if (e_ != hipSuccess) {                            \
            gd::note_hip_error(e_);                        \
            return GD_EHIP;                                \
        }                                                  \
    } while (0)

}  // namespace gd
