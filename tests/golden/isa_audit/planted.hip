// Kernels for the tests of the ISA coverage audit (Section 4.3: every load and store of a
// sandboxed kernel goes through the fence).  They are compiled to assembly text and
// audited, never linked into the library and never launched.  k_planted_ok uses the
// fence on every access; each of the others forgets it once, in the way its name
// says, and the audit has to report exactly that access.
#include "../../../paper_2401_09290_amd/csrc/fence.hpp"

namespace gd {

struct planted_args {
    uint64_t x;
    uint64_t y;
    uint64_t n;
};

// y[i] = 2 * x[i], every access fenced (address checking: tested, refused threads stop)
template <int V>
__global__ void k_planted_ok(planted_args p, FenceArgs fa)
{
    const Fence<V> F(fa);
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= p.n) return;
    const uint64_t a = p.x + 4 * i, b = p.y + 4 * i;
    if (!F.template inside<4>(a)) { F.fault(); return; }
    const float v = F.template ld<float>(a);
    if (!F.template inside<4>(b)) { F.fault(); return; }
    F.template st<float>(b, 2.0f * v);
}

// the store goes to the tenant's raw pointer
template <int V>
__global__ void k_planted_raw_store(planted_args p, FenceArgs fa)
{
    const Fence<V> F(fa);
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= p.n) return;
    const uint64_t a = p.x + 4 * i, b = p.y + 4 * i;
    if (!F.template inside<4>(a)) { F.fault(); return; }
    const float v = F.template ld<float>(a);
    *(GD_GLOBAL float *)b = 2.0f * v;
}

// address checking: the store's address is tested, but against the load's array
template <int V>
__global__ void k_planted_wrong_test(planted_args p, FenceArgs fa)
{
    const Fence<V> F(fa);
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= p.n) return;
    const uint64_t a = p.x + 4 * i, b = p.y + 4 * i;
    if (!F.template inside<4>(a)) { F.fault(); return; }
    const float v = F.template ld<float>(a);
    if (V == V_CHECK) *(GD_GLOBAL float *)b = 2.0f * v;
    else F.template st<float>(b, 2.0f * v);
}

// a wave-uniform element of tenant memory read without the fence (the compiler may use a scalar load)
template <int V>
__global__ void k_planted_uniform_read(planted_args p, FenceArgs fa)
{
    const Fence<V> F(fa);
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= p.n) return;
    const float s = *(const GD_GLOBAL float *)p.x;
    const uint64_t b = p.y + 4 * i;
    if (!F.template inside<4>(b)) { F.fault(); return; }
    F.template st<float>(b, s);
}

// a contiguous array read 16 bytes per lane through the per-array form, but from the raw pointer: the first byte was
// never fenced and the array never tested (under the hardware-checked rule the descriptor still bounds the access)
template <int V>
__global__ void k_planted_raw_tile(planted_args p, FenceArgs fa)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const Fence<V> F(fa);
    const uint64_t q0 = (uint64_t)blockIdx.x * blockDim.x;
    if (q0 + threadIdx.x >= p.n) return;
    const uint32_t lane_off = Fence<V>::template tile_lane_offset<1024>(16 * threadIdx.x);
    u32x4 v = F.template ld_tile16<u32x4>(p.x + 16 * q0, lane_off);
    F.tile_wait(v);
    const uint64_t b = p.y + 16 * (q0 + threadIdx.x);
    if (!F.template inside<16>(b)) { F.fault(); return; }
    F.template st<u32x4>(b, v);
}

#define GD_PLANT(V)                                                        \
    template __global__ void k_planted_ok<V>(planted_args, FenceArgs);        \
    template __global__ void k_planted_raw_store<V>(planted_args, FenceArgs); \
    template __global__ void k_planted_wrong_test<V>(planted_args, FenceArgs); \
    template __global__ void k_planted_uniform_read<V>(planted_args, FenceArgs); \
    template __global__ void k_planted_raw_tile<V>(planted_args, FenceArgs);
GD_PLANT(1)
GD_PLANT(2)
GD_PLANT(3)
GD_PLANT(4)
GD_PLANT(5)

}  // namespace gd
