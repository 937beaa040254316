// Device-side address fence for gfx950 kernels.
//
// Paper, Listing 1 and Section 4.3: every sandboxed kernel gets two extra
// parameters (partition base and mask), keeps them in two registers, and runs
//     addr = (addr AND mask) OR base
// on the final effective address in front of every global load and store.
// Here the two parameters arrive in the kernarg segment, so they live in SGPRs,
// and the fence is folded into the address arithmetic of each access:
//
//   V_BIT32  partition <= 4 GiB.  The fence keeps only address bits below the
//            mask, so the offset inside the partition is
//            lo32(addr) & mask32 -- one v_and_b32 -- and the OR with the base
//            is done by the global_load/store "SGPR base + 32-bit VGPR offset"
//            addressing mode (base is size-aligned, so OR == ADD).
//   V_BIT64  partition >= 4 GiB.  Then mask_lo = 0xFFFFFFFF and base_lo = 0, so
//            only the high word needs the AND/OR (two VALU ops).
//   V_NONE   native kernel: plain global pointer, no fence (Section 4.2.3).
//   V_MOD    Section 4.4's modulo fence, base + (addr - base) % size, for partitions
//            of any size and alignment: the 64-bit remainder is taken with a
//            multiply-high by a reciprocal the host precomputes per partition (the
//            paper's extra parameter holding 1/size), corrected to be exact.
//   V_CHECK  Section 4.4's address checking: the access proceeds unchanged if it
//            lies inside [base, base+size), otherwise the logical thread stops and
//            the tenant's fault counter (manager-owned memory) is incremented.
//
// Width rule: an access of W bytes also clears the low log2(W) address bits, so
// the whole access lies inside the partition (for naturally aligned addresses
// this is exactly the paper's rule).  The mask with those bits cleared is
// wave-uniform and is computed on the scalar unit.
//
// Rules for kernels using this header:
//   * every global access of tenant data goes through Fence::ld / Fence::st with
//     the FINAL address of that access (never index off a fenced pointer);
//   * a vector access (8/16 bytes) is only issued on an address the kernel has
//     established to be naturally aligned, so it equals the per-element fence;
//   * LDS and registers are not fenced (Section 3: not reachable by other
//     tenants); kernarg loads are not tenant-addressable.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace gd {

enum Variant : int { V_NONE = 0, V_BIT32 = 1, V_BIT64 = 2, V_MOD = 3, V_CHECK = 4, V_COUNT = 5 };

// The extra kernel parameters.  Listing 1's two (base, mask) are all the bitwise
// fence uses; the other rules of Section 4.4 reuse `mask` for the partition size
// and add the reciprocal (modulo) or the fault counter (checking).
struct FenceArgs {
    uint64_t base;
    uint64_t mask;      // bitwise: size - 1.  modulo, checking: size in bytes
    uint64_t magic;     // modulo: floor(2^64 * (2^shift - size) / size) + 1
    uint32_t shift;     // modulo: ceil(log2(size))
    uint32_t tenant;    // checking: slot of the launching tenant in the fault counters
    uint64_t faults;    // checking: device address of the uint64 fault counters, outside the pool
};

#define GD_GLOBAL __attribute__((address_space(1)))

// The AND of the 32-bit fence as one explicit VALU instruction (mask in an SGPR).
// Written as an instruction so that the optimiser cannot widen it back to 64 bits,
// which would lose the "SGPR base + 32-bit VGPR offset" addressing mode.
__device__ __forceinline__ uint32_t fence_and32(uint32_t addr_lo, uint32_t mask_lo)
{
    uint32_t off;
    asm("v_and_b32 %0, %1, %2" : "=v"(off) : "s"(mask_lo), "v"(addr_lo));
    return off;
}

template <int V>
struct Fence {
    uint64_t base;
    uint64_t mask;
    uint64_t magic;
    uint32_t shift;
    uint32_t tenant;
    uint64_t faults;

    static constexpr bool CHECKED = (V == V_CHECK);

    __device__ __forceinline__ explicit Fence(const FenceArgs &f)
        : base(f.base), mask(f.mask), magic(f.magic), shift(f.shift), tenant(f.tenant), faults(f.faults) {}

    // Address checking (V_CHECK only; every other rule lets all accesses through, the
    // fence having made them safe): is the whole W-byte access inside the partition?
    template <int W>
    __device__ __forceinline__ bool inside(uint64_t raw) const
    {
        if constexpr (V == V_CHECK) return raw - base <= mask - W;     // mask holds the size; wrap-around makes addr < base fail
        else return true;
    }

    // One violation: count it for the tenant.  The counter is manager-owned memory.
    __device__ __forceinline__ void fault() const
    {
        if constexpr (V == V_CHECK)
            __hip_atomic_fetch_add((GD_GLOBAL unsigned long long *)(faults + 8 * (uint64_t)tenant), 1ULL,
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }

    // The fenced address of a W-byte access to `raw` (what the probe kernel reports).
    template <int W>
    __device__ __forceinline__ uint64_t address(uint64_t raw) const
    {
        if constexpr (V == V_NONE || V == V_CHECK) {
            return raw;
        } else if constexpr (V == V_MOD) {
            // n mod d for any 64-bit n (Granlund-Montgomery division by an invariant):
            // q = (t + ((n - t) >> 1)) >> (shift - 1) with t = mulhi(magic, n).
            const uint64_t n = raw - base, d = mask;
            const uint64_t t = __umul64hi(magic, n);
            const uint64_t q = (t + ((n - t) >> 1)) >> (shift - 1);
            const uint64_t r = n - q * d;
            return base + (r & ~(uint64_t)(W - 1));
        } else if constexpr (V == V_BIT32) {
            const uint32_t m = (uint32_t)mask & ~(uint32_t)(W - 1);
            return base + (uint64_t)fence_and32((uint32_t)raw, m);
        } else {
            const uint32_t lo = (uint32_t)raw & ~(uint32_t)(W - 1);
            const uint32_t hi = ((uint32_t)(raw >> 32) & (uint32_t)(mask >> 32)) | (uint32_t)(base >> 32);
            return ((uint64_t)hi << 32) | lo;
        }
    }

    // STREAM = true marks data that is touched once (contiguous streams): the access
    // carries the nontemporal hint so that it does not displace reusable lines.
    template <typename T, bool STREAM = false>
    __device__ __forceinline__ T ld(uint64_t raw) const
    {
        const GD_GLOBAL T *ptr;
        if constexpr (V == V_BIT32) {
            const uint32_t m = (uint32_t)mask & ~(uint32_t)(sizeof(T) - 1);
            const uint32_t off = fence_and32((uint32_t)raw, m);
            ptr = (const GD_GLOBAL T *)((const GD_GLOBAL char *)base + off);
        } else {
            ptr = (const GD_GLOBAL T *)address<sizeof(T)>(raw);
        }
        if constexpr (STREAM) return __builtin_nontemporal_load(ptr);
        else return *ptr;
    }

    // A fenced address kept for a later access: the 32-bit offset inside the
    // partition for V_BIT32, the full address otherwise.
    using Handle = typename std::conditional<V == V_BIT32, uint32_t, uint64_t>::type;

    // A fenced address for dma16_unordered(), made from a wave-uniform 64-bit part
    // and a 32-bit per-lane byte offset.  The unfenced build keeps the two apart --
    // scalar base plus lane offset is an addressing mode of the copy instruction, so a
    // native kernel spends no vector instruction on the address -- and every fenced
    // build forms the sum and fences it (32-bit rule: in 32-bit arithmetic).
    struct Split { uint64_t s; uint32_t v; };
    using SplitHandle = typename std::conditional<V == V_NONE, Split, Handle>::type;

    template <int W>
    __device__ __forceinline__ SplitHandle fenced_split(uint64_t uniform_part, uint32_t lane_off) const
    {
        if constexpr (V == V_NONE) {
            return Split{uniform_part, lane_off};
        } else if constexpr (V == V_BIT32) {
            const uint32_t m = (uint32_t)mask & ~(uint32_t)(W - 1);
            return fence_and32((uint32_t)uniform_part + lane_off, m);
        } else {
            return address<W>(uniform_part + lane_off);
        }
    }

    // global -> LDS copy of 16 bytes per lane from an address fenced_split<16>()
    // produced, as an instruction the compiler does not model.  The compiler
    // orders every LDS read it cannot tell apart from an earlier global -> LDS copy
    // behind s_waitcnt vmcnt(0), which drains a software pipeline that keeps copies
    // in flight across basic blocks.  Issued this way the copy is invisible to that
    // bookkeeping: the caller owns the s_waitcnt vmcnt and the workgroup barrier
    // between the copy and the first read of its data.  `lds_addr` is the
    // wave-uniform LDS byte address lane 0 lands at; M0 carries it (one wait state
    // between the write of M0 and the copy).  M0 is a reserved register the compiler
    // does not track through inline asm: use this only in kernels where nothing else
    // depends on M0 (no compiler-issued LDS copies, no indexed register moves).
    //
    // OFF (64) selects the second half of the 128-byte line the handle points into.
    // It is applied to the fenced address -- through the scalar base for the 32-bit
    // rule, by setting bit 6 of the address otherwise -- which is the fence of the
    // final address only if the caller guarantees that the raw address the handle was
    // made from is a multiple of 128 plus less than 64: then bit 6 of the fenced
    // address is clear, adding 64 carries into nothing, and
    // fenced(raw) + 64 == fenced(raw + 64) (bitwise rule: the mask of a partition of at
    // least 4 KiB keeps the low 12 bits; modulo rule: base and size are multiples of
    // 256).  The instruction's own offset field is not used: it would move the LDS
    // side of the copy as well.
    template <int OFF = 0>
    __device__ __forceinline__ void dma16_unordered(SplitHandle h, uint32_t lds_addr) const
    {
        static_assert(OFF == 0 || OFF == 64, "only the two halves of a 128-byte line");
        if constexpr (V == V_NONE) {
            const uint64_t b = h.s + OFF;
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                         :
                         : "s"(lds_addr), "v"(h.v), "s"(b)
                         : "memory");
        } else if constexpr (V == V_BIT32) {
            const uint64_t b = base + OFF;                  // wave-uniform, loop-invariant
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                         :
                         : "s"(lds_addr), "v"(h), "s"(b)
                         : "memory");
        } else {
            const uint64_t a = h | (uint64_t)OFF;
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                         :
                         : "s"(lds_addr), "v"(a)
                         : "memory");
        }
    }

    template <typename T, bool STREAM = false>
    __device__ __forceinline__ void st(uint64_t raw, T v) const
    {
        GD_GLOBAL T *ptr;
        if constexpr (V == V_BIT32) {
            const uint32_t m = (uint32_t)mask & ~(uint32_t)(sizeof(T) - 1);
            const uint32_t off = fence_and32((uint32_t)raw, m);
            ptr = (GD_GLOBAL T *)((GD_GLOBAL char *)base + off);
        } else {
            ptr = (GD_GLOBAL T *)address<sizeof(T)>(raw);
        }
        if constexpr (STREAM) __builtin_nontemporal_store(v, ptr);
        else *ptr = v;
    }
};

// Launch helper for kernels built for all five variants.
#define GD_LAUNCH_VARIANT5(variant, KERNEL, grid, block, stream, ...)                           \
    do {                                                                                        \
        switch (variant) {                                                                      \
        case gd::V_NONE:  hipLaunchKernelGGL((KERNEL<gd::V_NONE>), grid, block, 0, stream, __VA_ARGS__); break;  \
        case gd::V_BIT32: hipLaunchKernelGGL((KERNEL<gd::V_BIT32>), grid, block, 0, stream, __VA_ARGS__); break; \
        case gd::V_BIT64: hipLaunchKernelGGL((KERNEL<gd::V_BIT64>), grid, block, 0, stream, __VA_ARGS__); break; \
        case gd::V_MOD:   hipLaunchKernelGGL((KERNEL<gd::V_MOD>), grid, block, 0, stream, __VA_ARGS__); break;   \
        case gd::V_CHECK: hipLaunchKernelGGL((KERNEL<gd::V_CHECK>), grid, block, 0, stream, __VA_ARGS__); break; \
        default: return GD_ENOKERNEL;                                                           \
        }                                                                                       \
    } while (0)

// Launch helper: instantiate KERNEL for the variant chosen on the host (no checking build).
#define GD_LAUNCH_VARIANT(variant, KERNEL, grid, block, stream, ...)                            \
    do {                                                                                        \
        switch (variant) {                                                                      \
        case gd::V_NONE:  hipLaunchKernelGGL((KERNEL<gd::V_NONE>), grid, block, 0, stream, __VA_ARGS__); break;  \
        case gd::V_BIT32: hipLaunchKernelGGL((KERNEL<gd::V_BIT32>), grid, block, 0, stream, __VA_ARGS__); break; \
        case gd::V_BIT64: hipLaunchKernelGGL((KERNEL<gd::V_BIT64>), grid, block, 0, stream, __VA_ARGS__); break; \
        case gd::V_MOD:   hipLaunchKernelGGL((KERNEL<gd::V_MOD>), grid, block, 0, stream, __VA_ARGS__); break;   \
        default: return GD_ENOKERNEL;                                                           \
        }                                                                                       \
    } while (0)

}  // namespace gd
