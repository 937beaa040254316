"""Pins for oracle/host_model.py: what the paper and the mathematics fix.

Nothing here calls the HIP library.
"""
import itertools
import random

import pytest

from oracle import host_model as hm

KiB = 1024


# ---------------------------------------------------------------------------
# Section 4.3 worked example
# ---------------------------------------------------------------------------

def test_mask_and_end_match_printed_example(golden):
    (base, size, end, mask), = golden("section4_3_mask_example.txt")
    base, size, end, mask = int(base, 16), int(size), int(end, 16), int(mask, 16)
    assert hm.partition_end(base, size) == end
    assert hm.partition_mask(base, size) == mask


def test_illegal_address_in_previous_partition_lands_in_own(golden):
    # Fig. 4: an address aimed at the partition in front is redirected into the
    # kernel's own partition at the same offset.
    (base, size, end, _), = golden("section4_3_mask_example.txt")
    base, size, end = int(base, 16), int(size), int(end, 16)
    other = base - size + 0x123456
    assert hm.fence(other, base, size) == base + 0x123456
    assert hm.fence(end + 1, base, size) == base            # one past the end wraps to the start
    assert hm.fence(end, base, size) == end


# ---------------------------------------------------------------------------
# Brute force on a tiny pool
# ---------------------------------------------------------------------------

TINY_BASE = 0x40000          # 256 KiB: aligned to the largest partition
TINY_BYTES = 64 * KiB
TINY_SIZES = [4 * KiB, 32 * KiB, 8 * KiB, 4 * KiB, 16 * KiB]


@pytest.fixture(scope="module")
def tiny_table():
    table = hm.carve(TINY_BASE, TINY_BYTES, TINY_SIZES)
    assert table is not None
    return table


def test_carve_tiny_pool_is_disjoint_aligned_inside_and_tight(tiny_table):
    owner = {}
    for t, (b, s) in enumerate(tiny_table):
        assert s == TINY_SIZES[t]
        assert b % s == 0
        assert TINY_BASE <= b and b + s <= TINY_BASE + TINY_BYTES
        for a in range(b, b + s, 256):
            assert a not in owner
            owner[a] = t
    assert len(owner) * 256 == sum(TINY_SIZES) == TINY_BYTES


@pytest.mark.parametrize("width", hm.ACCESS_WIDTHS)
def test_fence_confines_every_address_around_the_tiny_pool(tiny_table, width):
    lo, hi = TINY_BASE - 2 * TINY_BYTES, TINY_BASE + 3 * TINY_BYTES
    for (base, size) in tiny_table:
        end = hm.partition_end(base, size)
        for a in range(lo, hi):
            f = hm.fence(a, base, size, width)
            # whole footprint inside the tenant's own partition
            assert base <= f and f + width - 1 <= end
            # an access that already lies inside, naturally aligned, is unchanged
            if a % width == 0 and base <= a and a + width - 1 <= end:
                assert f == a
            # fencing twice changes nothing
            assert hm.fence(f, base, size, width) == f
            # the fence only ever drops address bits: same offset modulo the size
            assert (f - (a - a % width)) % size == 0


def test_bitwise_fence_equals_modulo_definition(tiny_table):
    # Section 4.4 states the modulo form as the same fencing without the
    # alignment requirement; for size-aligned partitions the two must agree on
    # every 64-bit address.
    rnd = random.Random(1)
    for (base, size) in tiny_table:
        probes = list(range(TINY_BASE - TINY_BYTES, TINY_BASE + 2 * TINY_BYTES, 7))
        probes += [0, 1, hm.U64, hm.U64 - 1, 1 << 63, (1 << 63) - 1, base - 1, base + size]
        probes += [rnd.getrandbits(64) for _ in range(20000)]
        for a in probes:
            assert hm.fence(a, base, size) == hm.fence_modulo(a, base, size)


def test_unaligned_base_would_alter_in_bounds_addresses():
    # A base that is not size-aligned breaks "in-bounds unchanged": this is why
    # partitions must be aligned to their size (the paper's example base is).
    size, base = 4096, 4096 + 256
    inside = base + 0x100
    assert ((inside & (size - 1)) | base) != inside
    with pytest.raises(AssertionError):
        hm.fence(inside, base, size)


def test_modulo_fence_with_width_keeps_whole_access_inside_odd_partitions():
    # Section 4.4: no power of two, no alignment.  Brute force on small odd partitions.
    for base, size in ((256 * 7, 256 * 3), (256 * 100, 256 * 17), (4096, 4096)):
        inside = set(range(base, base + size))
        for a in range(base - 2 * size, base + 3 * size, 3):
            for w in hm.ACCESS_WIDTHS:
                f = hm.fence_modulo(a, base, size, w)
                assert all(q in inside for q in (f, f + w - 1))
                if a % w == 0 and a in inside and a + w - 1 in inside:
                    assert f == a
                if a >= base:
                    assert (f - (a - a % w)) % size == 0 or (a - base) % size % w != 0


def test_carve_flex_is_disjoint_ordered_and_inside():
    rnd = random.Random(2)
    for _ in range(300):
        sizes = [256 * rnd.randint(16, 400) for _ in range(rnd.randint(1, 8))]
        pool_base = 256 * rnd.randint(1, 1000) + rnd.choice([0, 8])
        table = hm.carve_flex(pool_base, sum(sizes) + 256, sizes)
        assert table is not None
        owner = {}
        for t, (b, s) in enumerate(table):
            assert s == sizes[t] and b % 256 == 0 and pool_base <= b and b + s <= pool_base + sum(sizes) + 256
            for a in range(b, b + s, 256):
                assert a not in owner
                owner[a] = t
        assert [b for b, _ in table] == sorted(b for b, _ in table)      # tenant order = address order
        assert hm.carve_flex(pool_base, sum(sizes) - 256, sizes) is None


def test_fence_on_64bit_extremes():
    base, size = 0x7FA2D0000000, 1 << 24
    for a in (0, hm.U64, 1 << 63, 0xFFFF_FFFF_0000_0000, 0x0000_0000_FFFF_FFFF):
        f = hm.fence(a, base, size)
        assert f == base + (a % size)
    # partitions larger than 4 GiB: bits 32 and up of the offset survive
    base, size = 0x7F0000000000, 1 << 34
    a = base + (1 << 33) + 12
    assert hm.fence(a, base, size, 4) == a
    assert hm.fence(a + size, base, size, 4) == a


def test_width_aware_fence_vs_start_only_fence():
    # With the start-only rule a 16-byte access fenced to the last 4 bytes of
    # the partition would spill 12 bytes into the neighbour.
    base, size = 1 << 20, 1 << 12
    a = base + 2 * size - 4
    assert hm.fence(a, base, size, 1) == base + size - 4
    assert hm.fence(a, base, size, 16) == base + size - 16


# ---------------------------------------------------------------------------
# Address checking (Section 4.4)
# ---------------------------------------------------------------------------

def test_check_access_is_set_inclusion(tiny_table):
    base, size = tiny_table[2]
    inside = set(range(base, base + size))
    for a in range(base - 64, base + size + 64):
        for w in hm.ACCESS_WIDTHS:
            assert hm.check_access(a, base, size, w) == all(q in inside for q in range(a, a + w))


# ---------------------------------------------------------------------------
# Transfer range check (Section 4.2.2)
# ---------------------------------------------------------------------------

def test_check_copy_is_set_inclusion_on_tiny_partition():
    base, size = 0x3000, 0x1000
    inside = set(range(base, base + size))
    step = 64
    for p in range(base - 2 * size, base + 3 * size, step):
        for n in itertools.chain(range(0, 2 * size + step, step), (1, 3, size - 1, size + 1)):
            want = all(q in inside for q in (p, p + n - 1)) if n else (base <= p <= base + size)
            assert hm.check_copy(base, size, p, n) == want, (hex(p), n)


def test_check_copy_edges():
    base, size = 0x7FA2D0000000, 1 << 24
    assert hm.check_copy(base, size, base, size)
    assert not hm.check_copy(base, size, base, size + 1)
    assert not hm.check_copy(base, size, base - 1, 1)
    assert hm.check_copy(base, size, base + size - 1, 1)
    assert not hm.check_copy(base, size, base + size - 1, 2)
    assert hm.check_copy(base, size, base + size, 0)
    assert not hm.check_copy(base, size, base + size + 1, 0)
    # a range that would wrap the 64-bit address space is never inside
    assert not hm.check_copy(base, size, hm.U64 - 3, 8)
    assert not hm.check_copy(base, size, base + 16, hm.U64)


# ---------------------------------------------------------------------------
# Carving: properties that hold for any power-of-two request
# ---------------------------------------------------------------------------

def test_carve_random_requests_pack_tightly():
    # Power-of-two blocks placed by decreasing size into a pool aligned to the
    # largest block never leave a gap (buddy property): the carve must succeed
    # whenever the sizes sum to at most the pool, and occupy one contiguous run.
    rnd = random.Random(7)
    for _ in range(300):
        sizes = [1 << rnd.randint(12, 20) for _ in range(rnd.randint(1, 12))]
        biggest = max(sizes)
        pool_base = biggest * rnd.randint(1, 9)
        pool_bytes = sum(sizes)
        table = hm.carve(pool_base, pool_bytes, sizes)
        assert table is not None
        spans = sorted(table)
        for (b, s), size in zip(table, sizes):
            assert s == size and b % s == 0
        for (b0, s0), (b1, _) in zip(spans, spans[1:]):
            assert b0 + s0 == b1
        assert spans[0][0] == pool_base and spans[-1][0] + spans[-1][1] == pool_base + pool_bytes
        assert hm.carve(pool_base, pool_bytes - 1, sizes) is None


def test_carve_misaligned_pool_needs_slack():
    size = 1 << 16
    assert hm.carve(size + 4096, size, [size]) is None
    (b, s), = hm.carve(size + 4096, 2 * size, [size])
    assert b == 2 * size and s == size


def test_attach_detach_never_moves_other_tenants():
    rnd = random.Random(3)
    pool = hm.Pool(1 << 24, 1 << 24, [1 << 20, 1 << 22, 1 << 21])
    for _ in range(200):
        before = list(pool.table)
        live = [t for t, r in enumerate(pool.table) if r]
        if live and rnd.random() < 0.5:
            t = rnd.choice(live)
            assert pool.detach(t)
            before[t] = None
        else:
            size = 1 << rnd.randint(12, 22)
            t = pool.attach(size)
            if t is None:
                continue
            if t == len(before):
                before.append(None)
            assert before[t] is None
            before[t] = pool.table[t]
            b, s = pool.table[t]
            assert b % s == 0 and s == size
        assert pool.table == before
        rows = sorted(r for r in pool.table if r)
        for (b0, s0), (b1, _) in zip(rows, rows[1:]):
            assert b0 + s0 <= b1
        for (b, s) in rows:
            assert pool.pool_base <= b and b + s <= pool.pool_base + pool.pool_bytes


# ---------------------------------------------------------------------------
# Allocator model
# ---------------------------------------------------------------------------

def test_first_fit_against_byte_map():
    # Brute force: keep an occupancy map per 256-byte granule and check that
    # every allocation is the lowest aligned free run, never overlaps, stays
    # inside the partition; freeing everything makes the whole partition
    # allocatable again in one piece.
    rnd = random.Random(11)
    base, size = 1 << 20, 64 * KiB
    heap = hm.FirstFit(base, size)
    busy = [False] * (size // 256)
    live = {}
    for _ in range(3000):
        if live and rnd.random() < 0.45:
            p = rnd.choice(sorted(live))
            assert heap.free(p)
            for g in range((p - base) // 256, (p - base + live.pop(p)) // 256):
                busy[g] = False
            assert not heap.free(p)                 # double free is refused
            continue
        nbytes = rnd.randint(1, 6000)
        align = 1 << rnd.randint(0, 12)
        p = heap.alloc(nbytes, align)
        need = -(-nbytes // 256)
        eff_align = max(align, 256)
        want = None
        for g in range(len(busy) - need + 1):
            if (base + g * 256) % eff_align == 0 and not any(busy[g:g + need]):
                want = base + g * 256
                break
        assert p == want
        if p is not None:
            live[p] = need * 256
            for g in range((p - base) // 256, (p - base) // 256 + need):
                busy[g] = True
    for p in sorted(live):
        assert heap.free(p)
    assert heap.alloc(size, 256) == base
    assert heap.alloc(1, 256) is None
    assert heap.alloc(0) is None and heap.alloc(16, 3) is None
