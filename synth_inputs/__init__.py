"""Seeded synthetic inputs shared by the tests, the benchmark and the CPU oracle.

This module holds none of the method's arithmetic: no fence, no partition
placement, no kernel maths.  It only draws arrays (values, indices, offsets,
partition sizes) with the shapes and distributions of the five benchmark
configurations.  Pointers and partition geometry are passed in as plain
integers where a distribution is defined relative to them.

Random numbers: NumPy ``Generator(PCG64(seed))`` with
``seed = 20240109 + 1000 * config + tenant`` (plus ``10**6 * part`` for the
chunks of a large array).  The inputs stand in for the DRAM-resident ML kernels
the paper measured; no item of any dataset is reproduced.
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np

SEED0 = 20240109
MiB = 1 << 20
GiB = 1 << 30


def rng(config, tenant=0, part=0):
    return np.random.Generator(np.random.PCG64(SEED0 + 1000 * config + tenant + 10**6 * part))


# ---- values -----------------------------------------------------------------

def uniform_f32(g, n, lo=-1.0, hi=1.0):
    return (g.random(n, dtype=np.float32) * np.float32(hi - lo) + np.float32(lo)).astype(np.float32)


def normal_f32(g, n):
    return g.standard_normal(n, dtype=np.float32)


def fill_chunked(out, config, tenant, kind, lo=-1.0, hi=1.0, chunk=1 << 24, threads=8):
    """Fill a large float32 array chunk by chunk, each chunk from its own seeded
    stream, on a few threads (NumPy's generators release the GIL)."""
    n = out.size
    parts = [(p, s, min(s + chunk, n)) for p, s in enumerate(range(0, n, chunk))]

    def work(job):
        p, s, e = job
        g = rng(config, tenant, p + 1)
        out[s:e] = uniform_f32(g, e - s, lo, hi) if kind == "uniform" else normal_f32(g, e - s)

    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(work, parts))
    return out


def f32_to_bf16_bits(x):
    """Round float32 values to bfloat16 (ties to even); returns the uint16 patterns.
    Used to produce bfloat16 *inputs*; NaNs do not occur in the synthetic data."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def bf16_bits_to_f32(h):
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


# ---- configuration 1: indexed saxpy, 1 % of offsets out of range ---------------

def c1_offsets(g, n, y_ptr, part_base, part_size, frac=0.01, reach=16 * MiB):
    """int32 element offsets: identity, except that ``round(frac*n)`` positions
    (chosen without replacement) are replaced so that the byte address
    ``y_ptr + 4*off`` is uniform (4-byte aligned) over the ``reach`` bytes in
    front of the partition and the ``reach`` bytes behind it."""
    off = np.arange(n, dtype=np.int64)
    k = int(round(frac * n))
    where = g.choice(n, size=k, replace=False)
    slot = g.integers(0, 2 * reach // 4, size=k, dtype=np.int64) * 4
    target = np.where(slot < reach, part_base - reach + slot, part_base + part_size + (slot - reach))
    off[where] = (target - y_ptr) // 4
    assert np.all(np.abs(off) < 2**31)
    return off.astype(np.int32), np.sort(where)


# ---- configuration 2: gather / scatter with 64-bit indices ----------------------

def c2_indices(g, n, table_elems, frac=0.001, oob_hi=1 << 30):
    """int64 indices uniform over the table; ``round(frac*n)`` positions uniform in
    ``[table_elems, oob_hi)`` instead (out of bounds)."""
    idx = g.integers(0, table_elems, size=n, dtype=np.int64)
    k = int(round(frac * n))
    where = g.choice(n, size=k, replace=False)
    idx[where] = g.integers(table_elems, oob_hi, size=k, dtype=np.int64)
    return idx, np.sort(where)


# ---- configuration 5: mixed tenants ----------------------------------------------

def c5_partition_sizes(g, n=16, lo_log2=28, hi_log2=33, budget=200 * GiB):
    """Power-of-two partition sizes in [256 MiB, 8 GiB]; redrawn until at least one
    is 1 GiB or more and the sum fits the budget."""
    while True:
        sizes = [1 << int(e) for e in g.integers(lo_log2, hi_log2 + 1, size=n)]
        if max(sizes) >= GiB and sum(sizes) <= budget:
            return sizes


def c5_indices_i32(g, n, table_elems, frac=0.005, oob_hi=1 << 31):
    idx = g.integers(0, table_elems, size=n, dtype=np.int64)
    k = int(round(frac * n))
    where = g.choice(n, size=k, replace=False)
    idx[where] = g.integers(table_elems, oob_hi, size=k, dtype=np.int64)
    return idx.astype(np.int32), np.sort(where)


# ---- canaries --------------------------------------------------------------------

def chase_table(g, footprint_bytes, line=128):
    """uint32 table for the pointer chase: one entry per ``line`` bytes of the footprint is in use, and the
    used entries form ONE random cycle (entry -> index of the next used entry), so that a walk of any length
    visits a new cache line at every step and the whole footprint before it repeats.  Unused entries hold
    their own index.  Returns (table, index of a used entry to start from)."""
    per = line // 4
    slots = footprint_bytes // line
    assert slots >= 2 and footprint_bytes // 4 <= 1 << 32
    order = g.permutation(slots).astype(np.int64)                 # visiting order of the lines
    tab = np.arange(footprint_bytes // 4, dtype=np.uint32)
    tab[order * per] = (np.roll(order, -1) * per).astype(np.uint32)
    return tab, int(order[0] * per)


def canary_pattern(nbytes, byte=0xA5):
    return np.full(nbytes, byte, dtype=np.uint8)


def address_canary(n_words, salt=0):
    """64-bit words that depend on their position (a multiplicative hash of the
    index), so that a misplaced block copy is noticed as well as a stray store."""
    i = np.arange(n_words, dtype=np.uint64) + np.uint64(salt)
    with np.errstate(over="ignore"):
        z = (i + np.uint64(0x9E3779B97F4A7C15)) * np.uint64(0xBF58476D1CE4E5B9)
        z ^= z >> np.uint64(31)
    return z
