"""Pins for oracle/gd_oracle.c: its fence against the Python model and the
paper's example, its kernels against textbook NumPy routines on in-bounds
inputs, and against a per-byte Python retelling plus confinement on tiny pools
when accesses are out of bounds.  Nothing here calls the HIP library.
"""
import math
import random
import struct

import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import host_model as hm
from oracle import kernels as ok

KiB = 1024
BASE = 0x7FA2D0000000            # Section 4.3's example base, 16 MiB aligned


def make_pool(sizes, fill=0, pool_base=BASE):
    table = hm.carve(pool_base, sum(sizes), sizes)
    pool = ok.SimPool(pool_base, sum(sizes), fill)
    return pool, table


# ---------------------------------------------------------------------------
# fence
# ---------------------------------------------------------------------------

def test_c_fence_matches_printed_example(golden):
    (base, size, end, mask), = golden("section4_3_mask_example.txt")
    base, size, end = int(base, 16), int(size), int(end, 16)
    assert ok.fence(base, size, end + 1) == base
    assert ok.fence(base, size, base - 1) == end
    assert ok.fence(base, size, base - size + 0xABCDE) == base + 0xABCDE
    assert ok.fence(base, size, end) == end


@pytest.mark.parametrize("width", hm.ACCESS_WIDTHS)
def test_c_fence_equals_python_model_everywhere_on_tiny_pool(width):
    sizes = [4 * KiB, 32 * KiB, 8 * KiB, 4 * KiB, 16 * KiB]
    pool_base, pool_bytes = 0x40000, 64 * KiB
    table = hm.carve(pool_base, pool_bytes, sizes)
    addrs = np.arange(pool_base - 2 * pool_bytes, pool_base + 3 * pool_bytes, dtype=np.uint64)
    for (base, size) in table:
        got = ok.fence_array(base, size, addrs, width)
        want = (addrs & np.uint64((size - 1) & ~(width - 1))) | np.uint64(base)
        assert np.array_equal(got, want)
        # spot check the vector expression itself against the integer model
        for a in addrs[::997]:
            assert ok.fence(base, size, int(a), width) == hm.fence(int(a), base, size, width)
        assert got.min() >= base and got.max() + width - 1 <= base + size - 1


def test_c_fence_modes_on_random_64bit_addresses():
    rnd = random.Random(5)
    for _ in range(20000):
        size = 1 << rnd.randint(12, 40)
        base = size * rnd.randint(1, 1 << 10)
        a = rnd.getrandbits(64)
        w = rnd.choice(hm.ACCESS_WIDTHS)
        assert ok.fence(base, size, a, w, ok.MODE_BITWISE) == hm.fence(a, base, size, w)
        assert ok.fence(base, size, a, 1, ok.MODE_MODULO) == hm.fence_modulo(a, base, size)
        assert ok.fence(base, size, a, 1, ok.MODE_MODULO) == ok.fence(base, size, a, 1, ok.MODE_BITWISE)
        chk = ok.fence(base, size, a, w, ok.MODE_CHECK)
        assert (chk == a) == hm.check_access(a, base, size, w)
        assert chk in (a, hm.U64)
        assert ok.fence(base, size, a, w, ok.MODE_NONE) == a


@pytest.mark.parametrize("width", hm.ACCESS_WIDTHS)
def test_c_modulo_fence_with_width_against_integer_arithmetic(width):
    """Section 4.4's modulo rule with the width reading: the remainder is rounded down
    to a multiple of the access width.  The expected value is written out in Python
    integers (floor division, no bit tricks) next to the Python model's own value."""
    # every address around a tiny pool of odd-sized, 256-byte aligned partitions
    for (base, size) in ((0x40000, 4096 + 256), (0x41100, 4096 + 3 * 256), (0x43000, 7 * 256 + 4096)):
        for a in range(base - 2 * size - 7, base + 3 * size + 7):
            want = base + ((a - base) % (1 << 64)) % size // width * width   # the subtraction wraps at 2^64
            got = ok.fence(base, size, a, width, ok.MODE_MODULO)
            assert got == want == hm.fence_modulo(a, base, size, width)
            assert base <= got and got + width <= base + size
    # random 64-bit addresses, sizes up to 2^40 that are multiples of 256 but not powers of two
    rnd = random.Random(11 + width)
    for _ in range(20000):
        size = 256 * rnd.randint(17, 1 << 32)
        base = 256 * rnd.randint(1, 1 << 30)
        a = rnd.getrandbits(64)
        want = base + ((a - base) % (1 << 64)) % size // width * width
        assert ok.fence(base, size, a, width, ok.MODE_MODULO) == want == hm.fence_modulo(a, base, size, width)


def test_modulo_mode_accepts_unaligned_odd_sized_partitions():
    base, size = 1000, 300            # Section 4.4: modulo needs no alignment
    for a in range(0, 5000):
        f = ok.fence(base, size, a, 1, ok.MODE_MODULO)
        assert base <= f < base + size
        if a >= base:                     # below the base the 64-bit subtraction wraps
            assert (f - a) % size == 0
        if base <= a < base + size:
            assert f == a


# ---------------------------------------------------------------------------
# bfloat16 rounding
# ---------------------------------------------------------------------------

def test_bf16_rounding_closed_forms_and_library():
    L = ok.lib()
    one = 0x3F80
    assert L.gdo_double_to_bf16(1.0) == one
    assert L.gdo_double_to_bf16(1.0 + 2.0**-8) == one             # tie -> even (down)
    assert L.gdo_double_to_bf16(1.0 + 3 * 2.0**-8) == one + 2     # tie -> even (up)
    assert L.gdo_double_to_bf16(1.0 + 2.0**-8 + 2.0**-40) == one + 1
    assert L.gdo_double_to_bf16(-2.5) == 0xC020
    assert L.gdo_double_to_bf16(0.0) == 0 and L.gdo_double_to_bf16(-0.0) == 0x8000
    assert L.gdo_double_to_bf16(1e40) == 0x7F80 and L.gdo_double_to_bf16(-1e40) == 0xFF80
    assert L.gdo_double_to_bf16(2.0**-133) == 0x0001               # smallest subnormal
    assert L.gdo_double_to_bf16(2.0**-134) == 0x0000               # tie to even -> 0
    assert L.gdo_double_to_bf16(1.5 * 2.0**-134) == 0x0001
    # float32 inputs: one rounding step either way, so torch's conversion agrees
    g = np.random.Generator(np.random.PCG64(3))
    x = np.concatenate([g.standard_normal(20000).astype(np.float32),
                        (g.standard_normal(2000) * 1e-39).astype(np.float32),
                        (g.standard_normal(2000) * 1e30).astype(np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([L.gdo_double_to_bf16(float(v)) for v in x], dtype=np.uint16)
    assert np.array_equal(got, want)
    assert np.array_equal(si.f32_to_bf16_bits(x), want)             # the input generator's rounding too
    for h in (0x0000, 0x3F80, 0xC020, 0x0001, 0x7F7F):
        f = struct.unpack("<f", struct.pack("<I", h << 16))[0]
        assert L.gdo_bf16_to_double(h) == f


# ---------------------------------------------------------------------------
# kernels on in-bounds inputs reduce to textbook routines
# ---------------------------------------------------------------------------

@pytest.fixture()
def one_tenant():
    pool, table = make_pool([1 << 20, 1 << 20], fill=0xA5)
    return pool, table[0], table[1]


@pytest.mark.parametrize("mode", [ok.MODE_NONE, ok.MODE_BITWISE, ok.MODE_MODULO, ok.MODE_CHECK])
def test_streaming_kernels_are_memcpy_and_axpy(one_tenant, mode):
    pool, row, other = one_tenant
    n = 50001
    g = si.rng(0)
    a, b, c = row[0], row[0] + 256 * KiB, row[0] + 512 * KiB
    vb, vc = si.uniform_f32(g, n), si.uniform_f32(g, n)
    pool.view(b, np.float32, n)[:] = vb
    pool.view(c, np.float32, n)[:] = vc
    before_other = pool.view(other[0], np.uint8, other[1]).copy()
    assert pool.run("copy", row, mode, a, b, n) == (0, 0, 0)
    assert np.array_equal(pool.view(a, np.float32, n), vb)
    s = -0.37
    assert pool.run("triad", row, mode, a, b, c, s, n) == (0, 0, 0)
    want = (vb.astype(np.float64) + s * vc.astype(np.float64)).astype(np.float32)
    assert np.array_equal(pool.view(a, np.float32, n), want)
    assert pool.view(a, np.float32, n + 1)[n] != want[-1]          # nothing past n written
    pool.run("store_tid", row, mode, a, 77, n)
    assert np.all(pool.view(a, np.uint32, n) == 77)
    assert np.array_equal(pool.view(other[0], np.uint8, other[1]), before_other)


def test_indexed_kernels_are_fancy_indexing(one_tenant):
    pool, row, _ = one_tenant
    n = 20000
    g = si.rng(0, 1)
    x, y, off, out = (row[0] + k * 128 * KiB for k in range(4))
    vx, vy = si.uniform_f32(g, n), si.uniform_f32(g, n)
    perm = g.permutation(n).astype(np.int32)
    pool.view(x, np.float32, n)[:] = vx
    pool.view(y, np.float32, n)[:] = vy
    pool.view(off, np.int32, n)[:] = perm
    alpha = 0.8125
    pool.run("saxpy_idx", row, ok.MODE_BITWISE, x, y, off, alpha, n)
    want = (alpha * vx.astype(np.float64) + vy.astype(np.float64)).astype(np.float32)
    assert np.array_equal(pool.view(y, np.float32, n), want)       # a permutation touches each once

    # gather, 64-bit and 32-bit indices (duplicates allowed)
    idx64 = g.integers(0, n, size=n, dtype=np.int64)
    idxp = row[0] + 512 * KiB
    pool.view(idxp, np.int64, n)[:] = idx64
    pool.run("gather32_i64", row, ok.MODE_BITWISE, out, x, idxp, n)
    assert np.array_equal(pool.view(out, np.float32, n), vx[idx64])
    pool.view(idxp, np.int32, n)[:] = idx64.astype(np.int32)
    pool.view(out, np.float32, n)[:] = 0
    pool.run("gather32_i32", row, ok.MODE_BITWISE, out, x, idxp, n)
    assert np.array_equal(pool.view(out, np.float32, n), vx[idx64])

    # scatter with unique indices
    pool.view(idxp, np.int64, n)[:] = perm.astype(np.int64)
    pool.run("scatter_f32_i64", row, ok.MODE_BITWISE, y, x, idxp, -1.0, n)
    want = np.empty(n, np.float32)
    want[perm] = -vx
    assert np.array_equal(pool.view(y, np.float32, n), want)


def test_negative_offsets_and_indices_are_signed(one_tenant):
    pool, row, _ = one_tenant
    n = 64
    x, y, off = row[0] + 4 * KiB, row[0] + 8 * KiB, row[0] + 12 * KiB
    pool.view(x - 256, np.float32, 128)[:] = np.arange(128, dtype=np.float32)
    pool.view(y - 256, np.float32, 128)[:] = 1000 + np.arange(128, dtype=np.float32)
    offs = -np.arange(n, dtype=np.int32)
    pool.view(off, np.int32, n)[:] = offs
    pool.run("saxpy_idx", row, ok.MODE_BITWISE, x, y, off, 2.0, n)
    got = pool.view(y - 256, np.float32, 128)
    for k in range(128):
        e = k - 64
        want = 2.0 * k + 1000 + k if -n < e <= 0 else 1000 + k
        assert got[k] == want


def test_gather_i32_sign_extends_negative_and_large_indices(one_tenant):
    """Signed 32-bit indices: the element address is tab + 4*idx with idx sign-extended to
    64 bits, then fenced.  Expected values come from NumPy indexing of the partition seen
    as an array of words, at word number ((tab - base)/4 + idx) mod (size/4)."""
    pool, row, _ = one_tenant
    base, size = row
    words = size // 4
    n = 4096
    g = si.rng(0, 7)
    pool.view(base, np.uint32, words)[:] = g.integers(0, 1 << 32, size=words, dtype=np.uint64).astype(np.uint32)
    tab, idxp, out = base + 300 * KiB, base + 512 * KiB, base + 768 * KiB
    idx = np.concatenate([
        g.integers(-(1 << 31), 0, size=n // 4, dtype=np.int64),          # negative
        g.integers(1 << 30, 1 << 31, size=n // 4, dtype=np.int64),       # above 2^30
        g.integers(-70000, 70000, size=n // 4, dtype=np.int64),          # around the table start
        np.array([-(1 << 31), (1 << 31) - 1, -1, 0], dtype=np.int64),
        g.integers(0, 1 << 16, size=n // 4 - 4, dtype=np.int64)]).astype(np.int32)
    assert (idx < 0).sum() > n // 4 and (idx.astype(np.int64) > (1 << 30)).sum() >= n // 4
    pool.view(idxp, np.int32, n)[:] = idx
    pool.view(out, np.uint32, n)[:] = 0
    image = pool.view(base, np.uint32, words).copy()
    for mode in (ok.MODE_BITWISE, ok.MODE_MODULO):
        esc, vio, wrapped = pool.run("gather32_i32", row, mode, out, tab, idxp, n)
        assert esc == 0 and vio == 0 and wrapped > n // 2
        word = ((tab - base) // 4 + idx.astype(np.int64)) % words          # floor modulo on signed values
        want = image.copy()                     # in element order: a load may hit a word of `out` written earlier
        for i in range(n):
            want[(out - base) // 4 + i] = want[word[i]]
        assert np.array_equal(pool.view(base, np.uint32, words), want)
        pool.view(out, np.uint32, n)[:] = 0
    # With a power-of-two partition below 2^34 bytes the fence masks away exactly the bits in which a
    # sign-extended and a zero-extended index differ.  Two settings where they do show:
    # (1) no fence: a small negative index reads in front of the table;
    small = -np.arange(1, n + 1, dtype=np.int32)
    pool.view(idxp, np.int32, n)[:] = small
    assert pool.run("gather32_i32", row, ok.MODE_NONE, out, tab, idxp, n) == (0, 0, 0)
    assert np.array_equal(pool.view(out, np.uint32, n), image[(tab - base) // 4 + small.astype(np.int64)])
    # (2) the modulo fence on a partition whose size does not divide 2^34 (Section 4.4: any size).
    odd_base, odd_size = base + 256, 900 * KiB + 256
    pool.view(idxp, np.int32, n)[:] = idx
    pool.view(out, np.uint32, n)[:] = 0
    before = pool.mem.copy()
    esc, vio, _ = pool.run("gather32_i32", (odd_base, odd_size), ok.MODE_MODULO, out, tab, idxp, n)
    assert esc == 0 and vio == 0
    mem_words = before.view(np.uint32)
    want, want_zext = [], []
    for k in idx.tolist():
        a = odd_base + ((tab + 4 * k - odd_base) % (1 << 64)) % odd_size // 4 * 4
        z = odd_base + ((tab + 4 * (k % (1 << 32)) - odd_base) % (1 << 64)) % odd_size // 4 * 4
        want.append(mem_words[(a - pool.pool_base) // 4])
        want_zext.append(mem_words[(z - pool.pool_base) // 4])
    # `out` and the index array lie inside this partition too: skip loads that hit words `out` already holds
    clean = np.array([not (out <= odd_base + ((tab + 4 * k - odd_base) % (1 << 64)) % odd_size < out + 4 * n)
                      for k in idx.tolist()])
    got = pool.view(out, np.uint32, n)
    assert clean.mean() > 0.9 and np.array_equal(got[clean], np.array(want, np.uint32)[clean])
    assert not np.array_equal(got[clean], np.array(want_zext, np.uint32)[clean])


def test_sum_matches_fsum(one_tenant):
    pool, row, _ = one_tenant
    n = 100003
    v = si.uniform_f32(si.rng(0, 2), n, 0.0, 1.0)
    src, out = row[0], row[0] + 512 * KiB
    pool.view(src, np.float32, n)[:] = v
    pool.run("sum_f32", row, ok.MODE_BITWISE, out, src, n)
    exact = math.fsum(float(t) for t in v)
    assert pool.view(out, np.float32, 1)[0] == np.float32(exact)
    assert abs(pool.run("sum_f32_exact", row, ok.MODE_BITWISE, src, n) - exact) <= 1e-12 * exact


def test_rmsnorm_matches_formula(one_tenant):
    pool, row, _ = one_tenant
    rows, cols, eps = 7, 384, 1e-6
    g = si.rng(0, 3)
    xb = si.f32_to_bf16_bits(si.normal_f32(g, rows * cols))
    gb = si.f32_to_bf16_bits(si.uniform_f32(g, cols, 0.5, 1.5))
    x, gain, y = row[0], row[0] + 64 * KiB, row[0] + 128 * KiB
    pool.view(x, np.uint16, rows * cols)[:] = xb
    pool.view(gain, np.uint16, cols)[:] = gb
    pool.run("rmsnorm_bf16", row, ok.MODE_BITWISE, y, x, gain, rows, cols, eps)
    xf = si.bf16_bits_to_f32(xb).astype(np.float64).reshape(rows, cols)
    gf = si.bf16_bits_to_f32(gb).astype(np.float64)
    ref = xf / np.sqrt((xf * xf).mean(axis=1, keepdims=True) + eps) * gf
    got = si.bf16_bits_to_f32(pool.view(y, np.uint16, rows * cols)).astype(np.float64).reshape(rows, cols)
    # the result is the nearest bfloat16: within half a unit in the last place
    assert np.all(np.abs(got - ref) <= 2.0**-8 * np.abs(ref) * (1 + 1e-12))
    # rows of unit gain have unit mean square up to the output rounding
    pool.view(gain, np.uint16, cols)[:] = 0x3F80
    pool.run("rmsnorm_bf16", row, ok.MODE_BITWISE, y, x, gain, rows, cols, 0.0)
    got = si.bf16_bits_to_f32(pool.view(y, np.uint16, rows * cols)).astype(np.float64).reshape(rows, cols)
    assert np.allclose((got * got).mean(axis=1), 1.0, rtol=5e-3)


@pytest.mark.parametrize("b_is_nk", [0, 1])
def test_gemm_matches_numpy_matmul(one_tenant, b_is_nk):
    pool, row, _ = one_tenant
    M, N, K = 13, 22, 37                 # all different: a swapped extent shows
    g = si.rng(0, 4)
    Ab = si.f32_to_bf16_bits(si.normal_f32(g, M * K))
    Bb = si.f32_to_bf16_bits(si.normal_f32(g, K * N))
    A, B, Cc = row[0], row[0] + 64 * KiB, row[0] + 128 * KiB
    Af = si.bf16_bits_to_f32(Ab).astype(np.float64).reshape(M, K)
    Bf = si.bf16_bits_to_f32(Bb).astype(np.float64).reshape(K, N)
    pool.view(A, np.uint16, M * K)[:] = Ab
    stored = Bb.reshape(K, N).T.copy().reshape(-1) if b_is_nk else Bb
    pool.view(B, np.uint16, K * N)[:] = stored
    pool.run("gemm_bf16", row, ok.MODE_BITWISE, Cc, A, B, M, N, K, b_is_nk, 0, M, 0, N)
    ref = Af @ Bf
    got = si.bf16_bits_to_f32(pool.view(Cc, np.uint16, M * N)).astype(np.float64).reshape(M, N)
    assert np.all(np.abs(got - ref) <= 2.0**-8 * np.abs(ref) + 1e-12)
    want_bits = torch.from_numpy(ref.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    # double -> float -> bfloat16 may differ from the single rounding in rare ties only
    assert np.mean(pool.view(Cc, np.uint16, M * N) != want_bits.reshape(-1)) < 0.01
    e = pool.run("gemm_bf16_entry", row, ok.MODE_BITWISE, A, B, N, K, b_is_nk, 5, 9)
    assert abs(e - ref[5, 9]) <= 1e-12 * max(1.0, abs(ref[5, 9]))
    # a slab request writes only the slab
    pool.view(Cc, np.uint16, M * N)[:] = 0
    pool.run("gemm_bf16", row, ok.MODE_BITWISE, Cc, A, B, M, N, K, b_is_nk, 2, 4, 3, 8)
    nz = pool.view(Cc, np.uint16, M * N).reshape(M, N) != 0
    assert nz[2:4, 3:8].all() and nz.sum() == 2 * 5


# ---------------------------------------------------------------------------
# out-of-bounds behaviour on tiny pools
# ---------------------------------------------------------------------------

def py_saxpy_idx(mem, pool_base, base, size, x, y, off, alpha, n):
    """Per-byte retelling of the indexed saxpy in Python integers (tiny inputs)."""
    def F(a):
        return hm.fence(a & hm.U64, base, size, 4) - pool_base
    for i in range(n):
        o, = struct.unpack_from("<i", mem, F(off + 4 * i))
        vx, = struct.unpack_from("<f", mem, F(x + 4 * o))
        vy, = struct.unpack_from("<f", mem, F(y + 4 * o))
        r = np.float32(alpha * float(vx) + float(vy))
        struct.pack_into("<f", mem, F(y + 4 * o), r)


def test_out_of_bounds_saxpy_wraps_into_own_partition_only():
    sizes = [16 * KiB, 16 * KiB, 32 * KiB]
    pool, table = make_pool(sizes, fill=0xA5, pool_base=1 << 20)
    g = si.rng(0, 5)
    for tenant in (0, 1):
        base, size = table[tenant]
        n = 1024
        x, y, off = base, base + 4 * KiB, base + 8 * KiB
        pool.view(x, np.float32, n)[:] = si.uniform_f32(g, n)
        pool.view(y, np.float32, n)[:] = si.uniform_f32(g, n)
        offs, where = si.c1_offsets(g, n, y, base, size, frac=0.05, reach=64 * KiB)
        pool.view(off, np.int32, n)[:] = offs
        snapshot = pool.mem.copy()
        twin = bytearray(snapshot.tobytes())
        esc, vio, wrapped = pool.run("saxpy_idx", table[tenant], ok.MODE_BITWISE, x, y, off, 0.5, n)
        assert esc == 0 and vio == 0 and wrapped >= 3 * len(where) - 8
        py_saxpy_idx(twin, pool.pool_base, base, size, x, y, off, 0.5, n)
        assert pool.mem.tobytes() == bytes(twin)
        lo, hi = base - pool.pool_base, base - pool.pool_base + size
        assert np.array_equal(pool.mem[:lo], snapshot[:lo]) and np.array_equal(pool.mem[hi:], snapshot[hi:])
        assert not np.array_equal(pool.mem[lo:hi], snapshot[lo:hi])


def test_unfenced_out_of_bounds_store_does_corrupt_the_neighbour():
    # What the fence is for: the same launch without it writes into tenant 1.
    sizes = [4 * KiB, 4 * KiB]
    pool, table = make_pool(sizes, fill=0xA5, pool_base=1 << 16)
    base, size = table[0]
    n = 2 * size // 4                                   # runs over the end of tenant 0
    pool.run("store_tid", table[0], ok.MODE_NONE, base, 0x11111111, n)
    assert np.all(pool.view(table[1][0], np.uint32, size // 4) == 0x11111111)
    pool.mem[:] = 0xA5
    esc, vio, wrapped = pool.run("store_tid", table[0], ok.MODE_BITWISE, base, 0x11111111, n)
    assert wrapped == n // 2 and esc == 0
    assert np.all(pool.view(table[1][0], np.uint8, size) == 0xA5)
    assert np.all(pool.view(base, np.uint32, size // 4) == 0x11111111)
    pool.mem[:] = 0xA5
    esc, vio, wrapped = pool.run("store_tid", table[0], ok.MODE_CHECK, base, 0x11111111, n)
    assert vio == n // 2 and wrapped == 0
    assert np.all(pool.view(table[1][0], np.uint8, size) == 0xA5)
    # leaving the simulated pool altogether is counted, not performed
    esc, _, _ = pool.run("store_tid", table[0], ok.MODE_NONE, base + 2 * size - 8, 1, 4)
    assert esc == 2


def test_store_through_foreign_pointer_is_redirected():
    # A tenant that passes another tenant's buffer as its own pointer reaches
    # only its own partition, at the same offsets.
    sizes = [8 * KiB, 8 * KiB]
    pool, table = make_pool(sizes, fill=0, pool_base=1 << 16)
    (b0, s0), (b1, s1) = table
    pool.run("store_tid", table[0], ok.MODE_BITWISE, b1 + 64, 9, 100)
    assert np.all(pool.view(b1, np.uint8, s1) == 0)
    assert np.all(pool.view(b0 + 64, np.uint32, 100) == 9)


def test_pointer_chase_walks_the_cycle_and_every_step_goes_through_the_rule():
    """Pins of the chase: a walk of as many steps as the table has lines in use is back at its start (the
    generator builds one cycle), any walk equals the plain Python iteration, and an entry that points outside
    the partition is wrapped (bitwise, modulo), stops the thread (checking) or reads as zero (hardware
    checking) -- each computed here by hand."""
    sizes = [64 * KiB, 64 * KiB]
    pool, table = make_pool(sizes, fill=0xA5, pool_base=1 << 20)
    base, size = table[1]
    tab_host, first = si.chase_table(si.rng(7, 1), 32 * KiB)
    slots = 32 * KiB // 128
    assert sorted(np.flatnonzero(tab_host != np.arange(tab_host.size))) == sorted(range(0, tab_host.size, 32))
    tab, out, clk = base, base + 40 * KiB, base + 41 * KiB
    pool.view(tab, np.uint32, tab_host.size)[:] = tab_host
    # one whole cycle; a partial walk against plain iteration; several threads
    pool.run("chase", table[1], ok.MODE_BITWISE, out, clk, tab, slots, first, 0, 1)
    assert pool.view(out, np.uint32, 1)[0] == first and pool.last == (0, 0, 0)
    assert np.all(pool.view(clk, np.uint64, 2) == 0)
    steps, threads, hop = 77, 5, 32
    pool.run("chase", table[1], ok.MODE_BITWISE, out, clk, tab, steps, first, hop, threads)
    for t in range(threads):
        i = first + t * hop
        for _ in range(steps):
            i = int(tab_host[i])
        assert pool.view(out, np.uint32, threads)[t] == i
    # the entry after `first` sends the walk 3 entries past the partition's end
    second = int(tab_host[first])
    third = int(tab_host[second])
    beyond = size // 4 + 3
    for mode, lands in ((ok.MODE_BITWISE, 3), (ok.MODE_MODULO, 3), (ok.MODE_HWCHECK, None), (ok.MODE_CHECK, None)):
        pool.view(tab, np.uint32, tab_host.size)[:] = tab_host
        pool.view(tab, np.uint32, tab_host.size)[second] = beyond
        pool.view(out, np.uint32, 1)[0] = 0xDEAD
        pool.run("chase", table[1], mode, out, clk, tab, 3, first, 0, 1)
        got = int(pool.view(out, np.uint32, 1)[0])
        if mode in (ok.MODE_BITWISE, ok.MODE_MODULO):
            # first -> second -> (beyond, wrapped to entry 3, which is unused and holds its own index) -> 3
            assert got == int(pool.view(tab, np.uint32, tab_host.size)[3]) == 3 and pool.last[2] == 1
        elif mode == ok.MODE_HWCHECK:
            # the load outside reads zero: the walk continues at entry 0
            assert got == 0 and pool.last[1] == 1
        else:
            assert got == 0xDEAD and pool.last[1] == 1          # the thread stopped: nothing stored
    assert third != 3


def test_fence_addrs_probe_and_scatter_wrap():
    sizes = [16 * KiB, 16 * KiB]
    pool, table = make_pool(sizes, fill=0xA5, pool_base=1 << 20)
    base, size = table[1]
    n = 512
    rnd = random.Random(9)
    raw = np.array([rnd.getrandbits(64) for _ in range(n)], dtype=np.uint64)
    src, dst = base, base + 8 * KiB
    pool.view(src, np.uint64, n)[:] = raw
    for w in hm.ACCESS_WIDTHS:
        pool.run("fence_addrs", table[1], ok.MODE_BITWISE, dst, src, w, n)
        want = [hm.fence(int(a), base, size, w) for a in raw]
        assert pool.view(dst, np.uint64, n).tolist() == want
    # scatter with far out-of-range 64-bit indices (only the low bits survive)
    idx = np.array([rnd.getrandbits(63) for _ in range(64)], dtype=np.int64)
    vals = np.arange(64, dtype=np.float32) + 1
    pool.mem[:] = 0
    idxp, srcp, tab = base + 4 * KiB, base + 8 * KiB, base
    pool.view(idxp, np.int64, 64)[:] = idx
    pool.view(srcp, np.float32, 64)[:] = vals
    snapshot = pool.mem.copy()
    pool.run("scatter_f32_i64", table[1], ok.MODE_BITWISE, tab, srcp, idxp, 1.0, 64)
    changed = np.flatnonzero(pool.mem != snapshot)
    assert changed.size and changed.min() >= base - pool.pool_base
    images = {hm.fence((tab + 4 * int(k)) & hm.U64, base, size, 4) for k in idx}
    assert {int(c) // 4 * 4 + pool.pool_base for c in changed} <= images


# ---------------------------------------------------------------------------
# address checking (Sections 4.3, 4.4) in the kernels whose threads share operands
# ---------------------------------------------------------------------------

def test_checking_mode_gemm_stops_exactly_the_threads_with_a_refused_operand():
    """Thread (m, n) reads row m of A and column n of B and writes C[m,n]; it returns at its
    first refused access.  Expected image and count are built from set inclusion in NumPy."""
    sizes = [16 * KiB, 16 * KiB]
    pool, table = make_pool(sizes, fill=0xA5, pool_base=1 << 20)
    base, size = table[0]
    end = base + size
    M, N, K = 9, 14, 24
    g = si.rng(0, 8)
    for b_is_nk in (1, 0):
        A = base - 2 * (3 * K - 5)                # rows 0..2 of A start in front of the partition
        if b_is_nk:
            B = end - 2 * (10 * K + 7)            # stored N x K: columns 10.. of B run past the end
            Cc = base + 6 * KiB + 2               # inside
        else:
            B = base + 4 * KiB
            Cc = end - 2 * (5 * N + 3)            # C runs past the end of the partition from row 5 on
        pool.mem[:] = 0xA5
        Ab = si.f32_to_bf16_bits(si.normal_f32(g, M * K))
        Bb = si.f32_to_bf16_bits(si.normal_f32(g, K * N))
        stored = Bb.reshape(K, N).T.copy().reshape(-1) if b_is_nk else Bb
        # place what fits; the simulated pool covers both partitions, so out-of-partition operands exist in memory
        lo = pool.pool_base
        for ptr, bits in ((A, Ab), (B, stored)):
            for i, h in enumerate(bits.tolist()):
                a = ptr + 2 * i
                if lo <= a < lo + sum(sizes) - 1:
                    pool.view(a, np.uint16, 1)[0] = h
        before = pool.mem.copy()
        esc, vio, wrapped = pool.run("gemm_bf16", table[0], ok.MODE_CHECK, Cc, A, B, M, N, K, b_is_nk, 0, M, 0, N)
        assert esc == 0 and wrapped == 0

        def inside(a):
            return base <= a and a + 2 <= end
        a_ok = [all(inside(A + 2 * (m * K + k)) for k in range(K)) for m in range(M)]
        b_ok = [all(inside(B + 2 * ((n * K + k) if b_is_nk else (k * N + n))) for k in range(K)) for n in range(N)]
        Af = si.bf16_bits_to_f32(Ab).astype(np.float64).reshape(M, K)
        Bf = si.bf16_bits_to_f32(Bb).astype(np.float64).reshape(K, N)
        ref = Af @ Bf
        want = before.copy()
        stopped = 0
        for m in range(M):
            for n in range(N):
                c_addr = Cc + 2 * (m * N + n)
                if a_ok[m] and b_ok[n] and inside(c_addr):
                    h = ok.lib().gdo_double_to_bf16(float(ref[m, n]))
                    want[c_addr - lo:c_addr - lo + 2] = np.frombuffer(struct.pack("<H", h), np.uint8)
                else:
                    stopped += 1
        assert 0 < stopped < M * N and not all(a_ok) and any(a_ok)
        assert vio == stopped
        diff = np.flatnonzero(pool.mem != want)
        # fp64 accumulation order may differ from NumPy's in the last bit of a tie: allow no more than that
        assert diff.size <= 2, diff
        assert np.array_equal(pool.mem[size:], before[size:])          # the neighbour is untouched


def test_checking_mode_rmsnorm_row_and_element_refusals():
    """A row of x that is not wholly inside stops all of that row's threads (each counted);
    a gain or an output element outside stops that one thread."""
    sizes = [16 * KiB, 16 * KiB]
    pool, table = make_pool(sizes, fill=0xA5, pool_base=1 << 20)
    base, size = table[0]
    end = base + size
    rows, cols, eps = 6, 40, 1e-6
    g = si.rng(0, 9)
    x = base - 2 * (cols + 7)                      # row 0 and part of row 1 lie in front of the partition
    gain = end - 2 * 33                            # gains 33.. are past the end
    y = base + 4 * KiB - 2 * (rows * cols - 25)    # harmless: inside
    y2 = end - 2 * (4 * cols + 11)                 # second run: the output leaves the partition in row 4
    xb = si.f32_to_bf16_bits(si.normal_f32(g, rows * cols))
    gb = si.f32_to_bf16_bits(si.uniform_f32(g, cols, 0.5, 1.5))
    lo = pool.pool_base
    for yy, gain in ((y, gain), (y2, base + 8 * KiB)):    # second run: gains inside, so the output cannot overwrite them
        pool.mem[:] = 0xA5
        for ptr, bits in ((x, xb), (gain, gb)):
            for i, h in enumerate(bits.tolist()):
                a = ptr + 2 * i
                if lo <= a < lo + sum(sizes) - 1:
                    pool.view(a, np.uint16, 1)[0] = h
        before = pool.mem.copy()
        esc, vio, wrapped = pool.run("rmsnorm_bf16", table[0], ok.MODE_CHECK, yy, x, gain, rows, cols, eps)
        assert esc == 0 and wrapped == 0

        def inside(a):
            return base <= a and a + 2 <= end
        xf = si.bf16_bits_to_f32(xb).astype(np.float64).reshape(rows, cols)
        gf = si.bf16_bits_to_f32(gb).astype(np.float64)
        want = before.copy()
        stopped = 0
        for r in range(rows):
            row_ok = all(inside(x + 2 * (r * cols + j)) for j in range(cols))
            inv = 1.0 / math.sqrt(float((xf[r] * xf[r]).sum()) / cols + eps)
            for j in range(cols):
                out_addr = yy + 2 * (r * cols + j)
                if row_ok and inside(gain + 2 * j) and inside(out_addr):
                    h = ok.lib().gdo_double_to_bf16(float(xf[r, j] * inv * gf[j]))
                    want[out_addr - lo:out_addr - lo + 2] = np.frombuffer(struct.pack("<H", h), np.uint8)
                else:
                    stopped += 1
        assert vio == stopped and 2 * cols < stopped < rows * cols
        diff = np.flatnonzero(pool.mem != want)
        assert diff.size <= 2, diff                                    # summation order: at most a last-bit tie
        assert np.array_equal(pool.mem[size:], before[size:])


# ---------------------------------------------------------------------------
# the OpenMP build (timing only) computes what the sequential build computes
# ---------------------------------------------------------------------------

def test_openmp_twin_equals_the_sequential_oracle_on_in_bounds_inputs():
    g = si.rng(0, 10)
    n, rows, cols, M, N, K = 200003, 33, 256, 40, 24, 64
    images = []
    for openmp in (False, True):
        pool, table = make_pool([4 << 20, 4 << 20], fill=0xA5)
        row = table[0]
        g = si.rng(0, 10)
        p = [row[0] + k * (1 << 20) // 2 * 1 for k in range(8)]        # eight 512 KiB slots
        pool.view(p[0], np.float32, 100000)[:] = si.uniform_f32(g, 100000)
        pool.view(p[1], np.float32, 100000)[:] = si.uniform_f32(g, 100000)
        idx = g.integers(0, 100000, size=60000, dtype=np.int64)
        pool.view(p[2], np.int64, 60000)[:] = idx
        run = lambda name, *a: pool.run(name, row, ok.MODE_BITWISE, *a, openmp=openmp)
        run("triad", p[3], p[0], p[1], 0.3, 100000)
        run("copy", p[4], p[3], 100000)
        run("gather32_i64", p[5], p[0], p[2], 60000)
        pool.view(p[2], np.int64, 60000)[:] = g.permutation(60000)
        run("scatter_f32_i64", p[6], p[1], p[2], -1.0, 60000)
        run("sum_f32", p[7], p[0], 100000)
        xb = si.f32_to_bf16_bits(si.normal_f32(g, rows * cols))
        pool.view(p[7] + 4096, np.uint16, rows * cols)[:] = xb
        pool.view(p[7] + 65536, np.uint16, cols)[:] = si.f32_to_bf16_bits(si.uniform_f32(g, cols, 0.5, 1.5))
        run("rmsnorm_bf16", p[7] + 131072, p[7] + 4096, p[7] + 65536, rows, cols, 1e-6)
        run("gemm_bf16", p[7] + 262144, p[7] + 4096, p[7] + 4096 + 2 * M * K, M, N, K, 1, 0, M, 0, N)
        assert pool.last == (0, 0, 0)
        images.append(pool.mem.copy())
    diff = np.flatnonzero(images[0] != images[1])
    # only the sum may differ (another order of additions), and only in its last bits
    assert diff.size <= 2 and all(0 <= d - (p[7] - pool.pool_base) < 4 for d in diff)
    assert ok.lib(True).gdo_threads() >= 1 and ok.lib(False).gdo_threads() == 1


# ---------------------------------------------------------------------------
# hardware-style address checking (mode 4)
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("width", hm.ACCESS_WIDTHS)
def test_hwcheck_confines_or_refuses_every_address(width):
    """Brute force around a tiny pool of odd-sized partitions: an access is either made wholly
    inside the own partition, at the address the plain formula gives, or refused; in-partition
    aligned addresses are unchanged; addresses 2^32 apart behave alike."""
    for (base, size) in ((0x40000, 4096 + 256), (0x41100, 4096 + 3 * 256)):
        for a in range(base - 2 * size - 7, base + 3 * size + 7):
            got = ok.fence(base, size, a, width, ok.MODE_HWCHECK)
            off = ((a - base) % (1 << 32)) // width * width
            want = base + off if off + width <= size else hm.U64
            assert got == want
            assert (hm.fence_hwcheck(a, base, size, width) or hm.U64) == want
            if got != hm.U64:
                assert base <= got and got + width <= base + size
            if base <= a and a + width <= base + size and a % width == 0:
                assert got == a
            assert ok.fence(base, size, a + (1 << 32), width, ok.MODE_HWCHECK) == got
            assert ok.fence(base, size, a + (5 << 32), width, ok.MODE_HWCHECK) == got


def test_hwcheck_kernels_read_zero_and_drop_stores_outside():
    """Triad whose arrays run over the end of the partition: loads outside read 0, stores outside are
    dropped, the loop goes on (no thread stops); the neighbour partition is untouched."""
    sizes = [16 * KiB, 16 * KiB]
    pool, table = make_pool(sizes, fill=0xA5, pool_base=1 << 20)
    base, size = table[0]
    end = base + size
    n = 1000
    g = si.rng(0, 11)
    a, b, c = end - 4 * 700, base + 4 * KiB, end - 4 * 400        # a: 700 inside, c: 400 inside
    vb, vc = si.uniform_f32(g, n), si.uniform_f32(g, 400)
    pool.view(b, np.float32, n)[:] = vb
    pool.view(c, np.float32, 400)[:] = vc
    before = pool.mem.copy()
    esc, vio, wrapped = pool.run("triad", table[0], ok.MODE_HWCHECK, a, b, c, 0.5, n)
    assert esc == 0 and wrapped == 0 and vio == (n - 400) + (n - 700)
    cc = np.concatenate([vc.astype(np.float64), np.zeros(n - 400)])
    want = (vb.astype(np.float64) + 0.5 * cc).astype(np.float32)
    # a's elements 300.. overwrite c's memory, but element j reads c[j] before anything stores there (j + 300 comes later)
    image = before.copy()
    image[a - pool.pool_base:a - pool.pool_base + 4 * 700] = want[:700].view(np.uint8)
    assert np.array_equal(pool.mem, image)                         # stores 700.. dropped, neighbour untouched
    # gather through indices far outside: value 0 where refused
    idx = np.array([0, 5, 1 << 20, -2048, (1 << 30) + 7, 9], dtype=np.int64)    # (1<<30)+7: offset 4*(2^30+7) mod 2^32 = 28 -> inside
    tab, idxp, out = base + 4 * KiB, base + 8 * KiB, base + 12 * KiB
    pool.view(idxp, np.int64, idx.size)[:] = idx
    pool.view(out, np.uint32, idx.size)[:] = 0x77777777
    pool.run("gather32_i64", table[0], ok.MODE_HWCHECK, out, tab, idxp, idx.size)
    t = pool.view(tab, np.uint32, 16).copy()
    assert pool.view(out, np.uint32, idx.size).tolist() == [t[0], t[5], 0, 0, t[7], t[9]]


def test_the_oracle_itself_is_free_of_undefined_behaviour():
    """The checker is C with wrap-around address arithmetic, shifts and type-punned pool bytes: rerun this file's
    pins on a build of oracle/gd_oracle.c under gcc's undefined-behaviour sanitizer (GDO_UBSAN=1 makes
    oracle/kernels.py load that build; the first finding aborts the run)."""
    import os
    import subprocess
    import sys
    if os.environ.get("GDO_UBSAN") == "1":
        pytest.skip("already running on the sanitizer build")
    probe = subprocess.run(["gcc", "-fsanitize=undefined", "-static-libubsan", "-x", "c", "-", "-o", os.devnull],
                           input="int main(void){return 0;}", capture_output=True, text=True)
    if probe.returncode != 0:
        pytest.skip("gcc's undefined-behaviour sanitizer runtime is not installed")
    run = subprocess.run([sys.executable, "-m", "pytest", os.path.abspath(__file__), "-q", "-x", "-p", "no:cacheprovider"],
                         env=dict(os.environ, GDO_UBSAN="1"), capture_output=True, text=True, timeout=900,
                         cwd=os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    assert run.returncode == 0, run.stdout[-3000:] + run.stderr[-3000:]
    assert "runtime error" not in run.stderr and " passed" in run.stdout
