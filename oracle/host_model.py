"""Host-side semantics of Guardian's partitioning and fencing, in plain Python ints.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).  Every function states the
passage of the paper it follows.  Addresses are unsigned 64-bit values held in
Python integers; nothing here touches memory.

Parity status: pinned (tests/test_oracle_host_model.py) by the worked example of
Section 4.3, by brute force over tiny pools, and by equality of the bitwise
fence with the modulo definition of Section 4.4.
"""

U64 = (1 << 64) - 1

ACCESS_WIDTHS = (1, 2, 4, 8, 16)
GRANULE = 256


def is_pow2(v):
    return v > 0 and (v & (v - 1)) == 0


# ---------------------------------------------------------------------------
# Partition bounds table (Section 4.2.1) and mask derivation (Section 4.3)
# ---------------------------------------------------------------------------

def partition_end(base, size):
    """Highest address of a partition (inclusive), Section 4.3 worked example."""
    return base + size - 1


def partition_mask(base, size):
    """Mask of a partition, from its highest address and its size (Section 4.3).

    The bits in which the highest address differs from the base are exactly the
    bits an in-partition offset may use; for a power-of-two size that is
    ``size - 1``.  Both forms are computed and must agree.
    """
    assert is_pow2(size) and base % size == 0
    m = partition_end(base, size) ^ base
    assert m == size - 1
    return m


def carve(pool_base, pool_bytes, sizes):
    """Split one reserved pool into one contiguous partition per tenant.

    Section 4.2.1: the manager reserves the memory and gives each tenant one
    contiguous block; Section 1 / 4.4: blocks are powers of two and aligned to
    their size.  The paper fixes no placement order; this build places tenants
    by decreasing size (ties by tenant number), each at the lowest
    size-aligned address of the pool that is still free.

    Returns a list ``[(base, size), ...]`` indexed by tenant, or ``None`` if
    the request does not fit.
    """
    table = [None] * len(sizes)
    order = sorted(range(len(sizes)), key=lambda t: (-sizes[t], t))
    for t in order:
        spot = lowest_free_aligned(pool_base, pool_bytes, [r for r in table if r], sizes[t])
        if spot is None:
            return None
        table[t] = (spot, sizes[t])
    return table


def lowest_free_aligned(pool_base, pool_bytes, taken, size):
    """Lowest ``a`` with ``a % size == 0``, ``[a, a+size)`` inside the pool and
    disjoint from every ``(base, size)`` in ``taken``; ``None`` if there is none.
    Also the rule for attaching a tenant to a pool that is already carved.
    """
    assert is_pow2(size)
    pool_end = pool_base + pool_bytes
    a = -(-pool_base // size) * size
    while a + size <= pool_end:
        clash = [b + s for (b, s) in taken if a < b + s and b < a + size]
        if not clash:
            return a
        a = -(-max(clash) // size) * size
    return None


# ---------------------------------------------------------------------------
# The fence (Listing 1 and Section 4.3) and its modulo definition (Section 4.4)
# ---------------------------------------------------------------------------

def fence(addr, base, size, width=1):
    """Bitwise address fence: AND with the mask, then OR with the base.

    Listing 1 applies the two operations, in this order, to the final
    effective address right before the access.  ``width`` is the access size
    in bytes: the paper fences the start address only, which on hardware that
    allows unaligned global accesses would let the last access of a partition
    straddle its end, so this build also clears the low ``log2(width)`` bits.
    For a naturally aligned address the result is the paper's rule exactly.
    """
    assert width in ACCESS_WIDTHS and 0 <= addr <= U64
    mask = partition_mask(base, size) & ~(width - 1) & U64
    return (addr & mask) | base


def fence_modulo(addr, base, size, width=1):
    """Section 4.4: ``base + ((addr - base) % size)``, subtraction in wrap-around
    64-bit arithmetic, ``%`` the non-negative remainder.  No alignment needed.
    ``width``: as for the bitwise fence, the low bits of the offset are cleared so
    that the whole access stays inside (base and size are multiples of the width)."""
    assert width in ACCESS_WIDTHS
    return base + ((((addr - base) & U64) % size) & ~(width - 1))


def carve_flex(pool_base, pool_bytes, sizes):
    """Partitions of arbitrary size for the modulo fence and address checking
    (Section 4.4: no power of two, no alignment to the size): tenants in order,
    each at the lowest 256-byte aligned address that is still free."""
    table = []
    for size in sizes:
        spot = lowest_free(pool_base, pool_bytes, table, size, GRANULE)
        if spot is None:
            return None
        table.append((spot, size))
    return table


def lowest_free(pool_base, pool_bytes, taken, size, align):
    pool_end = pool_base + pool_bytes
    a = -(-pool_base // align) * align
    while a + size <= pool_end:
        clash = [b + s for (b, s) in taken if a < b + s and b < a + size]
        if not clash:
            return a
        a = -(-max(clash) // align) * align
    return None


def check_access(addr, base, size, width=1):
    """Address checking (Section 4.4): is the whole access inside the partition?"""
    return base <= addr and addr + width - 1 <= partition_end(base, size)


def fence_hwcheck(addr, base, size, width=1):
    """Address checking as a GPU's buffer addressing performs it (this build's addition to
    Section 4.4's list of rules): the access is made at a 32-bit offset from the partition
    base, ``(addr - base) mod 2^32`` with the low bits of the width cleared, and refused
    (``None``) unless the whole access lies below the partition size.  Every access that is
    made lies inside the partition; addresses 4 GiB apart are not told apart."""
    assert width in ACCESS_WIDTHS and size < (1 << 32)
    off = ((addr - base) & 0xFFFFFFFF) & ~(width - 1)
    return base + off if off + width <= size else None


# ---------------------------------------------------------------------------
# Transfer range check (Section 4.2.2)
# ---------------------------------------------------------------------------

def check_copy(base, size, ptr, nbytes):
    """Accept a host-initiated copy/memset iff ``[ptr, ptr+nbytes)`` lies inside
    the caller's partition.  Half-open range: an empty range is accepted at any
    ``ptr`` in ``[base, base+size]``.  Only the partition bounds are consulted,
    never the live allocations (Section 5, "Buffer overflow")."""
    return base <= ptr and ptr + nbytes <= base + size


# ---------------------------------------------------------------------------
# In-partition allocator model (Section 4.2.1; policy is this build's)
# ---------------------------------------------------------------------------

class FirstFit:
    """Address-ordered first fit inside one partition, written the slow way.

    Section 4.2.1 only says that the intercepted malloc is served from the
    tenant's partition and that free marks the region free.  Policy chosen for
    determinism: sizes are rounded up to 256 bytes, alignment is a power of
    two of at least 256, and a request gets the lowest suitably aligned
    address whose range overlaps no live allocation.
    """

    def __init__(self, base, size):
        self.base, self.size = base, size
        self.live = {}          # start -> rounded size

    def alloc(self, nbytes, align=GRANULE):
        if nbytes <= 0 or not is_pow2(align):
            return None
        align = max(align, GRANULE)
        nbytes = -(-nbytes // GRANULE) * GRANULE
        p = -(-self.base // align) * align
        for start in sorted(self.live):
            if p + nbytes <= start:
                break
            stop = start + self.live[start]
            if stop > p:
                p = -(-stop // align) * align
        if p + nbytes > self.base + self.size:
            return None
        self.live[p] = nbytes
        return p

    def free(self, ptr):
        return self.live.pop(ptr, None) is not None


class Pool:
    """Partition bounds table with attach/detach, mirroring the manager's state
    (Section 4.2.1): per tenant ``(base, size)`` plus that tenant's allocator."""

    def __init__(self, pool_base, pool_bytes, sizes):
        self.pool_base, self.pool_bytes = pool_base, pool_bytes
        table = carve(pool_base, pool_bytes, sizes)
        if table is None:
            raise MemoryError("partitions do not fit the pool")
        self.table = list(table)
        self.heaps = [FirstFit(b, s) for (b, s) in table]

    def attach(self, size):
        taken = [r for r in self.table if r]
        spot = lowest_free_aligned(self.pool_base, self.pool_bytes, taken, size)
        if spot is None:
            return None
        slot = self.table.index(None) if None in self.table else len(self.table)
        if slot == len(self.table):
            self.table.append(None)
            self.heaps.append(None)
        self.table[slot] = (spot, size)
        self.heaps[slot] = FirstFit(spot, size)
        return slot

    def detach(self, tenant):
        if self.heaps[tenant].live:
            return False
        self.table[tenant] = None
        self.heaps[tenant] = None
        return True
