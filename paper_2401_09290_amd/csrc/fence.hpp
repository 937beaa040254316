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
//   V_BUF    address checking done by the memory pipeline: every access is a buffer
//            instruction through a descriptor {base, num_records = size} of the
//            tenant's partition (below 4 GiB), with the 32-bit offset
//            lo32(addr - base), low log2(W) bits cleared.  The hardware compares
//            offset + W with num_records: an access outside returns 0 (load) or is
//            dropped (store); nothing is counted and no thread stops.  Addresses
//            4 GiB apart share an offset, so this rule confines (every access lands
//            in the partition or nowhere) but does not detect every stray address.
//
// Width rule: an access of W bytes also clears the low log2(W) address bits, so
// the whole access lies inside the partition (for naturally aligned addresses
// this is exactly the paper's rule).  The mask with those bits cleared is
// wave-uniform and is computed on the scalar unit.
//
// Rules for kernels using this header:
//   * every global access of tenant data goes through Fence::ld / Fence::st with
//     the FINAL address of that access (never index off a fenced pointer) -- or
//     through the per-array form below: a kernel that has tested with whole_run()
//     that the fence maps an array to one contiguous range may fence its first
//     byte once (scalar_fence) and address it as fenced start + offset
//     (ld_tile16 / st_tile16 / dma16_unordered), which then IS the fence of
//     every final address;
//   * a vector access (8/16 bytes) is only issued on an address the kernel has
//     established to be naturally aligned, so it equals the per-element fence;
//   * LDS and registers are not fenced (Section 3: not reachable by other
//     tenants); kernarg loads are not tenant-addressable.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace gd {

enum Variant : int { V_NONE = 0, V_BIT32 = 1, V_BIT64 = 2, V_MOD = 3, V_CHECK = 4, V_BUF = 5, V_COUNT = 6 };

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

    // `count` violations (one per stopped logical thread): add them to the tenant's
    // counter.  The counter is manager-owned memory.
    __device__ __forceinline__ void fault(uint64_t count = 1) const
    {
        if constexpr (V == V_CHECK)
            __hip_atomic_fetch_add((GD_GLOBAL unsigned long long *)(faults + 8 * (uint64_t)tenant),
                                   (unsigned long long)count, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }

    // Address checking of a run of `bytes` consecutive bytes (an operand row): every
    // 2-, 4-, ... byte element of it is inside the partition iff the run is.
    __device__ __forceinline__ bool inside_run(uint64_t raw, uint64_t bytes) const
    {
        if constexpr (V == V_CHECK) return bytes <= mask && raw - base <= mask - bytes;
        else return true;
    }

    // The fenced address of a W-byte access to `raw` (what the probe kernel reports).
    template <int W>
    __device__ __forceinline__ uint64_t address(uint64_t raw) const
    {
        if constexpr (V == V_NONE || V == V_CHECK) {
            return raw;
        } else if constexpr (V == V_BUF) {
            const uint64_t off = buf_offset<W>(raw);
            return off + W <= mask ? base + off : ~(uint64_t)0;        // mask holds the size
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

    // The same for an access each lane makes on its own (ld, st, fenced).  Modulo rule: if every active
    // lane's access lies inside the partition -- one 64-bit compare and a wave-uniform branch -- the
    // remainder is the difference itself and the reciprocal arithmetic (about 25 vector instructions) is
    // skipped for the whole wavefront; a wavefront with any lane outside takes the exact path for all.
    template <int W>
    __device__ __forceinline__ uint64_t lane_address(uint64_t raw) const
    {
        if constexpr (V == V_MOD) {
            const uint64_t n = raw - base;
            if (__builtin_amdgcn_ballot_w64(n > mask - W) == 0) return base + (n & ~(uint64_t)(W - 1));   // mask holds the size
        }
        return address<W>(raw);
    }

    // ---- scalar tile fence ------------------------------------------------------------
    // A wavefront that accesses start + L, with `start` wave-uniform and the lane
    // offsets L all below TILE, can take the fence once, on the scalar unit: if the
    // fenced image of `start` has TILE bytes of the partition behind it, then adding L
    // carries into no masked bit and fence(start + L) == fence(start) + L for every
    // such L, exactly.  tile() tests that condition and gives the fenced start; when it
    // does not hold (a tenant pointer that wraps at the partition end inside this tile)
    // the caller takes its per-lane path.  `start` must be aligned to the width of the
    // accesses made through the tile, so that the width rule clears nothing.
    // The bitwise rules run Listing 1's two 64-bit instructions as they stand, on
    // SGPR pairs; the accesses then use the "SGPR base + 32-bit VGPR offset"
    // addressing mode with the lane offset as the offset (ld_tile / st_tile).
    template <int TILE>
    __device__ __forceinline__ uint64_t tile(uint64_t start, uint64_t &fenced) const
    {
        // Returns 0 if the tile is whole (see above), anything else if the fence splits it;
        // a caller with several tiles ORs the results and tests once.
        if constexpr (V == V_NONE) {
            fenced = start;
            return 0;
        } else if constexpr (V == V_BUF) {
            fenced = buf_offset<16>(start);          // offsets wrap at 2^32 by definition: a tile is never split
            return 0;
        } else if constexpr (V == V_CHECK) {
            fenced = start;
            return !inside<TILE>(start);
        } else if constexpr (V == V_MOD) {
            // a start that is inside the partition already is its own image: the division is skipped (scalar branch)
            if (start - base < mask) fenced = start;             // mask holds the size
            else fenced = address<1>(start);
            return !(fenced - base <= mask - TILE);
        } else {
            asm("s_and_b64 %0, %1, %2\n\ts_or_b64 %0, %0, %3" : "=&s"(fenced) : "s"(start), "s"(mask), "s"(base) : "scc");
            // offset + TILE - 1 <= mask, as "no bit above the mask" (scalar unit: no 64-bit ordered compare)
            return ((start & mask) + (TILE - 1)) & ~mask;
        }
    }

    // The same for a whole contiguous array of `bytes` bytes starting at `start` (both
    // wave-uniform): if whole_run() holds, the fence maps the array to ONE contiguous
    // range, i.e. fence(start + d) == fence(start) + d for every d < bytes, exactly.  A
    // kernel tests its streams once, fences each array's first byte once
    // (scalar_fence(start), on the scalar unit), and then addresses the array as
    // "fenced start + offset" like a native kernel: no fence instruction is left in
    // its loop, for any rule.
    __device__ __forceinline__ bool whole_run(uint64_t start, uint64_t bytes) const
    {
        if constexpr (V == V_NONE || V == V_BUF) return true;       // V_BUF: offsets wrap at 2^32 by definition
        else if constexpr (V == V_CHECK) return inside_run(start, bytes);
        else if constexpr (V == V_MOD) {
            const uint64_t image = (start - base < mask) ? start : address<1>(start);
            return bytes <= mask && image - base <= mask - bytes;
        }
        else return (((start & mask) + (bytes ? bytes - 1 : 0)) & ~mask) == 0;    // last byte's offset <= mask, in a form the scalar unit has
    }
    __device__ __forceinline__ uint64_t scalar_fence(uint64_t start) const
    {
        uint64_t fenced;
        (void)tile<16>(start, fenced);
        return fenced;
    }

    // The lane's byte offset inside a tile of TILE bytes, confined below TILE by an AND
    // with a constant (one instruction per kernel, not per access).  Callers may pass
    // stride * threadIdx.x: the AND also reduces it to the lane's offset in its wavefront.
    template <int TILE>
    static __device__ __forceinline__ uint32_t tile_lane_offset(uint32_t off)
    {
        static_assert((TILE & (TILE - 1)) == 0, "tile size must be a power of two");
        uint32_t r;
        asm("v_and_b32 %0, %1, %2" : "=v"(r) : "n"(TILE - 1), "v"(off));
        return r;
    }

    // 16-byte accesses through a tile: the instruction is written out, so that its
    // form -- fenced SGPR pair as the base, the confined lane offset as the 32-bit
    // offset -- does not depend on what the optimiser makes of the address
    // arithmetic.  The compiler does not count these loads: tile_wait() must stand
    // between a ld_tile16 and the first use of its result.
    // OFFS: a constant byte offset inside the tile, carried by the instruction (the tile
    // test covers every byte of the tile, so fenced + lane_off + OFFS stays inside).
    template <typename T, bool STREAM = false, int OFFS = 0>
    __device__ __forceinline__ T ld_tile16(uint64_t fenced, uint32_t lane_off) const
    {
        static_assert(sizeof(T) == 16 && OFFS >= 0 && OFFS < 4096, "one 16-byte vector per lane");
        if constexpr (V == V_BUF) return buf_load<T, STREAM>((uint32_t)fenced + lane_off + OFFS);
        T v;
        if constexpr (STREAM) asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3 nt" : "=v"(v) : "v"(lane_off), "s"(fenced), "n"(OFFS) : "memory");
        else asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3" : "=v"(v) : "v"(lane_off), "s"(fenced), "n"(OFFS) : "memory");
        return v;
    }

    // THROUGH (with STREAM): the nontemporal store is also written through at device scope ("sc1 nt").  Measured
    // on 1 GiB arrays of random values: copy 316.5 us against 320.4 us for "nt" alone (+1.2 %), triad unchanged
    // (479 us; a plain store: 512 us); on arrays of 64 to 256 MiB the triad is 1.5 to 7 % slower with it.  Used by
    // the copy.
    template <typename T, bool STREAM = false, bool THROUGH = false>
    __device__ __forceinline__ void st_tile16(uint64_t fenced, uint32_t lane_off, T v) const
    {
        static_assert(sizeof(T) == 16, "one 16-byte vector per lane");
        if constexpr (V == V_BUF) {
            buf_store<T, STREAM>((uint32_t)fenced + lane_off, v);
            return;
        }
        // s_nop 1: a store of more than 64 bits reads its data up to two wait states late, and the compiler, which
        // pads its own stores, does not see this one
        if constexpr (STREAM && THROUGH) asm volatile("global_store_dwordx4 %0, %1, %2 sc1 nt\n\ts_nop 1" : : "v"(lane_off), "v"(v), "s"(fenced) : "memory");
        else if constexpr (STREAM) asm volatile("global_store_dwordx4 %0, %1, %2 nt\n\ts_nop 1" : : "v"(lane_off), "v"(v), "s"(fenced) : "memory");
        else asm volatile("global_store_dwordx4 %0, %1, %2\n\ts_nop 1" : : "v"(lane_off), "v"(v), "s"(fenced) : "memory");
    }

    // All ld_tile16 issued so far have landed; the values pass through so that no use
    // of them can be scheduled in front of the wait.
    template <typename T>
    static __device__ __forceinline__ void tile_wait(T &a)
    {
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(a) : : "memory");
    }
    template <typename T>
    static __device__ __forceinline__ void tile_wait(T &a, T &b)
    {
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(a), "+v"(b) : : "memory");
    }
    // All but the youngest ld_tile16 have landed (they return in issue order): lets the arithmetic on the first
    // results run while the last load is still in flight.  Only in straight-line code, with the number of loads in
    // flight fixed: between a ld_tile16 and the wait that covers it the compiler must have no reason to touch the
    // load's registers (the ISA audit checks that no instruction does).
    template <typename T>
    static __device__ __forceinline__ void tile_wait_all_but_last(T &a, T &b)
    {
        asm volatile("s_waitcnt vmcnt(1)" : "+v"(a), "+v"(b) : : "memory");
    }
    // ---- V_BUF: the partition as a raw buffer --------------------------------------------
    // Descriptor words: base (48 bits), stride 0, num_records = size in bytes, and the
    // gfx9-family data-format word for untyped accesses.  Wave-uniform: built on the
    // scalar unit, once.
    __device__ __forceinline__ __amdgpu_buffer_rsrc_t descriptor() const
    {
        return __builtin_amdgcn_make_buffer_rsrc((void *)(uintptr_t)base, 0, (uint32_t)mask, 0x00020000);
    }
    template <int W>
    __device__ __forceinline__ uint32_t buf_offset(uint64_t raw) const
    {
        return ((uint32_t)raw - (uint32_t)base) & ~(uint32_t)(W - 1);
    }
    template <typename T, bool STREAM>
    __device__ __forceinline__ T buf_load(uint32_t off) const
    {
        constexpr int AUX = STREAM ? 2 : 0;                    // bit 1: nontemporal
        const __amdgpu_buffer_rsrc_t r = descriptor();
        if constexpr (sizeof(T) == 1) return __builtin_bit_cast(T, (uint8_t)__builtin_amdgcn_raw_buffer_load_b8(r, off, 0, AUX));
        else if constexpr (sizeof(T) == 2) return __builtin_bit_cast(T, (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(r, off, 0, AUX));
        else if constexpr (sizeof(T) == 4) return __builtin_bit_cast(T, (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(r, off, 0, AUX));
        else if constexpr (sizeof(T) == 8) return __builtin_bit_cast(T, __builtin_amdgcn_raw_buffer_load_b64(r, off, 0, AUX));
        else return __builtin_bit_cast(T, __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, AUX));
    }
    template <typename T, bool STREAM>
    __device__ __forceinline__ void buf_store(uint32_t off, T v) const
    {
        constexpr int AUX = STREAM ? 2 : 0;
        typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
        typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
        const __amdgpu_buffer_rsrc_t r = descriptor();
        if constexpr (sizeof(T) == 1) __builtin_amdgcn_raw_buffer_store_b8(__builtin_bit_cast(uint8_t, v), r, off, 0, AUX);
        else if constexpr (sizeof(T) == 2) __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(uint16_t, v), r, off, 0, AUX);
        else if constexpr (sizeof(T) == 4) __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, v), r, off, 0, AUX);
        else if constexpr (sizeof(T) == 8) __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2_t, v), r, off, 0, AUX);
        else __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, v), r, off, 0, AUX);
    }

    // STREAM = true marks data that is touched once (contiguous streams): the access
    // carries the nontemporal hint so that it does not displace reusable lines.
    template <typename T, bool STREAM = false>
    __device__ __forceinline__ T ld(uint64_t raw) const
    {
        if constexpr (V == V_BUF) return buf_load<T, STREAM>(buf_offset<sizeof(T)>(raw));
        const GD_GLOBAL T *ptr;
        if constexpr (V == V_BIT32) {
            const uint32_t m = (uint32_t)mask & ~(uint32_t)(sizeof(T) - 1);
            const uint32_t off = fence_and32((uint32_t)raw, m);
            ptr = (const GD_GLOBAL T *)((const GD_GLOBAL char *)base + off);
        } else {
            ptr = (const GD_GLOBAL T *)lane_address<sizeof(T)>(raw);
        }
        if constexpr (STREAM) return __builtin_nontemporal_load(ptr);
        else return *ptr;
    }

    // A fenced address kept for a later access: the 32-bit offset inside the
    // partition for V_BIT32, the full address otherwise.
    using Handle = typename std::conditional<V == V_BIT32, uint32_t, uint64_t>::type;

    // The fence now, the access later: fenced<W>(raw) is the Handle of a W-byte access to `raw`, st_fenced /
    // ld_fenced perform it.  A kernel with several data-dependent accesses per lane computes all its handles
    // first and pins them with keep_apart(), so that each sits in registers of its own: an instruction that
    // rewrites the address or data register of the memory instruction in front of it has to wait until that
    // one has read its operands, and behind a queue of random accesses that wait is long (measured on the
    // scatter: 998 us with one address register pair reused by four stores, 917 us with four pairs).
    template <int W>
    __device__ __forceinline__ Handle fenced(uint64_t raw) const
    {
        if constexpr (V == V_BIT32) return fence_and32((uint32_t)raw, (uint32_t)mask & ~(uint32_t)(W - 1));
        else if constexpr (V == V_BUF) return buf_offset<W>(raw);
        else return lane_address<W>(raw);
    }
    template <typename T>
    __device__ __forceinline__ void st_fenced(Handle h, T v) const
    {
        if constexpr (V == V_BUF) buf_store<T, false>((uint32_t)h, v);
        else if constexpr (V == V_BIT32) *(GD_GLOBAL T *)((GD_GLOBAL char *)base + h) = v;
        else *(GD_GLOBAL T *)h = v;
    }
    template <typename T>
    __device__ __forceinline__ T ld_fenced(Handle h) const
    {
        if constexpr (V == V_BUF) return buf_load<T, false>((uint32_t)h);
        else if constexpr (V == V_BIT32) return *(const GD_GLOBAL T *)((const GD_GLOBAL char *)base + h);
        else return *(const GD_GLOBAL T *)h;
    }
    // Four handles and four values live at once, i.e. in distinct registers (no instruction is emitted).
    template <typename T>
    static __device__ __forceinline__ void keep_apart(Handle &h0, Handle &h1, Handle &h2, Handle &h3, T &v0, T &v1, T &v2, T &v3)
    {
        asm volatile("" : "+v"(h0), "+v"(h1), "+v"(h2), "+v"(h3), "+v"(v0), "+v"(v1), "+v"(v2), "+v"(v3));
    }

    static __device__ __forceinline__ void keep_apart(Handle &h0, Handle &h1, Handle &h2, Handle &h3)
    {
        asm volatile("" : "+v"(h0), "+v"(h1), "+v"(h2), "+v"(h3));
    }

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
        } else if constexpr (V == V_BUF) {
            // the buffer offset of the sum: the uniform part's offset (scalar unit) plus the lane's
            return (uint64_t)((((uint32_t)uniform_part - (uint32_t)base) + lane_off) & ~(uint32_t)(W - 1));
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
    // between the write of M0 and the copy).  M0 is a register the compiler reserves
    // and does not track through inline asm (it rejects a clobber declaration for it):
    // use this only in kernels where nothing else depends on M0 (no compiler-issued
    // LDS copies, no indexed register moves).
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
        } else if constexpr (V == V_BUF) {
            // the same copy as a buffer instruction: the lane's offset is range-checked against the partition's
            // size by the memory pipeline, a lane outside delivers zeros to the LDS (measured: lane l lands in the
            // 16-byte slot l behind M0, as with the global form).  The partition base is a multiple of 256, so
            // bit 6 of the offset is bit 6 of the raw address and OFF can be ORed in as below.
            typedef uint32_t words_t __attribute__((ext_vector_type(4)));
            const words_t r = {(uint32_t)base, (uint32_t)(base >> 32) & 0xffffu, (uint32_t)mask, 0x00020000u};   // mask holds the size
            const uint32_t off = (uint32_t)h | (uint32_t)OFF;
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                         :
                         : "s"(lds_addr), "v"(off), "s"(r)
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
        if constexpr (V == V_BUF) {
            buf_store<T, STREAM>(buf_offset<sizeof(T)>(raw), v);
            return;
        }
        GD_GLOBAL T *ptr;
        if constexpr (V == V_BIT32) {
            const uint32_t m = (uint32_t)mask & ~(uint32_t)(sizeof(T) - 1);
            const uint32_t off = fence_and32((uint32_t)raw, m);
            ptr = (GD_GLOBAL T *)((GD_GLOBAL char *)base + off);
        } else {
            ptr = (GD_GLOBAL T *)lane_address<sizeof(T)>(raw);
        }
        if constexpr (STREAM) __builtin_nontemporal_store(v, ptr);
        else *ptr = v;
    }
};

}  // namespace gd
