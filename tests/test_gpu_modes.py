"""GPU parity for the two other bounds-checking rules of Section 4.4 -- the modulo
fence (partitions of any size and alignment) and address checking (an offending
logical thread stops and is counted) -- and for address checking done by the
memory pipeline (buffer instructions: an access outside reads zero or is dropped).
Same bars as test_gpu_parity.py; the fault counters must equal the oracle's
violation counts exactly.
"""
import numpy as np
import pytest
import torch

import paper_2401_09290_amd as gd
import synth_inputs as si
from harness import KiB, MiB, Rig, assert_bf16_close, rel_frobenius
from oracle import host_model as hm
from oracle import kernels as ok

pytestmark = pytest.mark.gpu


class FlexRig:
    """Device pool with partitions of arbitrary size, mirrored by the oracle."""

    def __init__(self, sizes, fill=0xA5, misalign=256 * 3):
        total = sum(sizes) + 4096
        self.buf = torch.empty(total + misalign, dtype=torch.uint8, device="cuda")
        self.base = self.buf.data_ptr() + misalign            # deliberately not aligned to anything large
        self.bytes = total
        self.dev = self.buf[misalign:misalign + total]
        self.dev.fill_(fill)
        self.pool = gd.gd_pool_create_flex(self.base, total, sizes)
        self.table = hm.carve_flex(self.base, total, sizes)
        for t, row in enumerate(self.table):
            assert gd.gd_partition_info(self.pool, t)[:2] == row
        self.heaps = [hm.FirstFit(b, s) for (b, s) in self.table]
        self.sim = ok.SimPool(self.base, total, fill)
        torch.cuda.synchronize()

    def alloc(self, t, nbytes):
        p = gd.gd_alloc(self.pool, t, nbytes)
        assert p == self.heaps[t].alloc(nbytes)
        return p

    def upload(self, t, ptr, arr):
        arr = np.ascontiguousarray(arr)
        assert gd.gd_check_copy(self.pool, t, ptr, arr.nbytes) == gd.GD_OK
        self.dev[ptr - self.base:ptr - self.base + arr.nbytes].copy_(torch.from_numpy(arr.view(np.uint8).reshape(-1)))
        self.sim.view(ptr, arr.dtype, arr.size)[:] = arr.reshape(-1)

    def download(self, ptr, dtype, count):
        n = count * np.dtype(dtype).itemsize
        return self.dev[ptr - self.base:ptr - self.base + n].cpu().numpy().view(dtype)

    def images_equal(self, skip=()):
        torch.cuda.synchronize()
        got, want = self.dev.cpu().numpy().copy(), self.sim.mem.copy()
        for (p, n) in skip:
            got[p - self.base:p - self.base + n] = 0
            want[p - self.base:p - self.base + n] = 0
        return np.array_equal(got, want)

    def close(self):
        gd.gd_pool_destroy(self.pool)
        self.buf = self.dev = self.sim = None
        torch.cuda.empty_cache()


def random_addresses(g, n, base, size):
    raw = g.integers(0, 1 << 63, size=n, dtype=np.uint64) * np.uint64(2) + g.integers(0, 2, size=n, dtype=np.uint64)
    raw[: n // 2] = np.uint64(base) + g.integers(0, 4 * size, size=n // 2, dtype=np.uint64) - np.uint64(2 * size)
    return raw


# ---------------------------------------------------------------------------
# modulo fence
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("width", [1, 4, 16])
def test_modulo_probe_agrees_with_bitwise_on_aligned_power_of_two_partitions(width):
    r = Rig([4 * MiB, 4 * MiB])
    try:
        g = si.rng(6, width)
        base, size = r.row(1)
        n = 30000
        raw = random_addresses(g, n, base, size)
        src, dst = r.alloc(1, 8 * n), r.alloc(1, 8 * n)
        r.upload(1, src, raw)
        r.launch(1, gd.GD_K_FENCE_ADDRS, gd.gd_args_fence_addrs(dst, src, n, width, 0), mode=gd.GD_FENCE_MODULO)
        got = r.download(dst, np.uint64, n)
        assert np.array_equal(got, ok.fence_array(base, size, raw, width, ok.MODE_MODULO))
        assert np.array_equal(got, ok.fence_array(base, size, raw, width, ok.MODE_BITWISE))
    finally:
        r.close()


def test_modulo_fence_on_partitions_of_odd_size_and_alignment():
    sizes = [3 * MiB + 256, 5 * MiB + 768, MiB + 256 * 17]
    r = FlexRig(sizes)
    try:
        g = si.rng(6, 50)
        for t, (base, size) in enumerate(r.table):
            assert size & (size - 1) and base % 4096                    # neither a power of two nor page aligned
            n = 20001
            raw = random_addresses(g, n, base, size)
            src, dst = r.alloc(t, 8 * n), r.alloc(t, 8 * n)
            r.upload(t, src, raw)
            for width in (1, 2, 4, 8, 16):
                gd.gd_launch_fenced(r.pool, t, gd.GD_K_FENCE_ADDRS, gd.gd_args_fence_addrs(dst, src, n, width, 0), mode=gd.GD_FENCE_MODULO)
                r.sim.run("fence_addrs", (base, size), ok.MODE_MODULO, dst, src, width, n)
                got = r.download(dst, np.uint64, n)
                assert np.array_equal(got, ok.fence_array(base, size, raw, width, ok.MODE_MODULO))
                assert got.min() >= base and got.max() + width <= base + size
            # whole wavefronts of addresses inside the partition (the per-lane rule's wave-uniform shortcut), the last
            # 64 bytes of the partition among them (inside or not, depending on the width), then mixed wavefronts
            inb = np.uint64(base) + g.integers(0, size - 16, size=n, dtype=np.uint64)
            inb[:64] = np.uint64(base + size) - np.arange(1, 65, dtype=np.uint64)
            inb[n // 2:] = raw[n // 2:]
            r.upload(t, src, inb)
            for width in (1, 2, 4, 8, 16):
                gd.gd_launch_fenced(r.pool, t, gd.GD_K_FENCE_ADDRS, gd.gd_args_fence_addrs(dst, src, n, width, 0), mode=gd.GD_FENCE_MODULO)
                r.sim.run("fence_addrs", (base, size), ok.MODE_MODULO, dst, src, width, n)
                assert np.array_equal(r.download(dst, np.uint64, n), ok.fence_array(base, size, inb, width, ok.MODE_MODULO)), width
            # a store loop twice as long as the partition, from a pointer in front of it: wraps, stays inside
            gd.gd_launch_fenced(r.pool, t, gd.GD_K_STORE_TID, gd.gd_args_store_tid(base - 1000 * 4, 2 * size // 4, 40 + t, 0), mode=gd.GD_FENCE_MODULO)
            r.sim.run("store_tid", (base, size), ok.MODE_MODULO, base - 1000 * 4, 40 + t, 2 * size // 4)
            assert r.images_equal(), f"tenant {t}"
        # arithmetic kernels through pointers that are off by whole partitions
        t = 1
        base, size = r.table[t]
        n = 100003
        bufs = [base + k * 512 * KiB for k in range(6)]
        a, b, c, idx, out = bufs[0], bufs[1], bufs[2], bufs[3], bufs[5]      # idx (8 bytes per element) takes two slots
        r.upload(t, b, si.uniform_f32(g, n))
        r.upload(t, c, si.uniform_f32(g, n))
        gd.gd_launch_fenced(r.pool, t, gd.GD_K_TRIAD, gd.gd_args_triad(a + 3 * size, b - size, c + size, n, 0.75, 0), mode=gd.GD_FENCE_MODULO)
        r.sim.run("triad", (base, size), ok.MODE_MODULO, a + 3 * size, b - size, c + size, 0.75, n)
        assert rel_frobenius(r.download(a, np.float32, n), r.sim.view(a, np.float32, n)) <= 1e-5
        assert r.images_equal(skip=[(a, 4 * n)])
        r.upload(t, a, r.sim.view(a, np.float32, n).copy())               # wrapped loads below may read `a`: same bits on both sides
        ix, where = si.c2_indices(g, n, n, frac=0.01, oob_hi=1 << 40)
        img = ok.fence_array(base, size, np.uint64(b) + (4 * ix[where]).astype(np.uint64), 4, ok.MODE_MODULO)
        ix[where[(img >= out) & (img < out + 4 * n)]] = 5                 # loads that would race with this launch's stores
        r.upload(t, idx, ix)
        gd.gd_launch_fenced(r.pool, t, gd.GD_K_GATHER32_I64, gd.gd_args_gather(out, b, idx, n), mode=gd.GD_FENCE_MODULO)
        r.sim.run("gather32_i64", (base, size), ok.MODE_MODULO, out, b, idx, n)
        assert r.sim.last[2] > 0.9 * len(where)
        assert r.images_equal()
    finally:
        r.close()


def test_modulo_scatter_and_indexed_saxpy_through_indices_that_wrap_whole_partitions():
    """Indices and offsets that are too large by whole multiples of the (odd) partition size: the modulo rule brings
    every such access back to the element an in-range index would have named (not so for negative ones: the rule
    works on the wrap-around difference, and 2^64 is no multiple of an odd size), so the launch is free of aliasing by
    construction, every wrapped access is counted by the oracle, and the whole image must match bit for bit
    (vector path and, through a misaligned index array, the per-element path)."""
    sizes = [3 * MiB + 256, 5 * MiB + 768]
    r = FlexRig(sizes)
    try:
        g = si.rng(6, 51)
        t = 1
        base, size = r.table[t]
        per = size // 4                                   # the partition in 4-byte elements (size is a multiple of 256)
        n = 50003
        for shift in (0, 8):                              # shift 8: the 64-bit index array is not 16-byte aligned
            src, dst, idx, x, y, off = (r.alloc(t, 4 * n), r.alloc(t, 4 * n), r.alloc(t, 8 * n + 16), r.alloc(t, 4 * n),
                                        r.alloc(t, 4 * n), r.alloc(t, 4 * n + 16))
            r.upload(t, src, si.uniform_f32(g, n))
            r.upload(t, dst, np.zeros(n, np.float32))
            k = g.permutation(n).astype(np.int64)
            far = g.choice(n, size=n // 20, replace=False)
            k[far] += g.integers(1, 1000, size=far.size) * per
            r.upload(t, idx + shift, k)
            gd.gd_launch_fenced(r.pool, t, gd.GD_K_SCATTER_F32_I64, gd.gd_args_scatter(dst, src, idx + shift, n, -2.0, 0), mode=gd.GD_FENCE_MODULO)
            r.sim.run("scatter_f32_i64", (base, size), ok.MODE_MODULO, dst, src, idx + shift, -2.0, n)
            assert r.sim.last[2] >= far.size and r.sim.last[0] == 0
            assert r.images_equal(), f"scatter, shift {shift}"
            o = np.arange(n, dtype=np.int64)
            o[far] += g.integers(1, 300, size=far.size) * per
            assert np.abs(o).max() < 1 << 31
            r.upload(t, x, si.uniform_f32(g, n))
            r.upload(t, y, si.uniform_f32(g, n))
            r.upload(t, off + shift // 2, o.astype(np.int32))
            gd.gd_launch_fenced(r.pool, t, gd.GD_K_SAXPY_IDX, gd.gd_args_saxpy_idx(x, y, off + shift // 2, n, 0.625, 0), mode=gd.GD_FENCE_MODULO)
            r.sim.run("saxpy_idx", (base, size), ok.MODE_MODULO, x, y, off + shift // 2, 0.625, n)
            assert r.sim.last[2] >= far.size and r.sim.last[0] == 0
            assert rel_frobenius(r.download(y, np.float32, n), r.sim.view(y, np.float32, n)) <= 1e-5
            assert r.images_equal(skip=[(y, 4 * n)]), f"saxpy, shift {shift}"
            r.upload(t, y, r.sim.view(y, np.float32, n).copy())
    finally:
        r.close()


def test_modulo_mode_rmsnorm_and_gemm_match_the_oracle():
    r = FlexRig([6 * MiB + 512, 2 * MiB + 256])
    try:
        g = si.rng(6, 60)
        base, size = r.table[0]
        rows, cols = 9, 2048
        x, y, gain = r.alloc(0, 2 * rows * cols), r.alloc(0, 2 * rows * cols), r.alloc(0, 2 * cols)
        r.upload(0, x, si.f32_to_bf16_bits(si.normal_f32(g, rows * cols)))
        r.upload(0, gain, si.f32_to_bf16_bits(si.uniform_f32(g, cols, 0.5, 1.5)))
        gd.gd_launch_fenced(r.pool, 0, gd.GD_K_RMSNORM_BF16, gd.gd_args_rmsnorm(y + size, x - size, gain, rows, cols, 1e-6, 0), mode=gd.GD_FENCE_MODULO)
        r.sim.run("rmsnorm_bf16", (base, size), ok.MODE_MODULO, y + size, x - size, gain, rows, cols, 1e-6)
        got, want = r.download(y, np.uint16, rows * cols), r.sim.view(y, np.uint16, rows * cols)
        assert_bf16_close(got, want, what="modulo rmsnorm")
        # (512, 256, 384): the per-array form of the DMA-ring kernel (operands mapped to one contiguous range each),
        # here through a pointer one partition too high and one that is not mapped contiguously (fallback per lane)
        for (M, N, K) in ((256, 256, 128), (512, 256, 384), (256, 512, 320), (100, 72, 40)):      # K = 320: the ring of K = 64 blocks
            A, B, Cc = r.alloc(0, 2 * M * K), r.alloc(0, 2 * K * N), r.alloc(0, 2 * M * N)
            r.upload(0, A, si.f32_to_bf16_bits(si.normal_f32(g, M * K) * np.float32(K ** -0.5)))
            r.upload(0, B, si.f32_to_bf16_bits(si.normal_f32(g, K * N)))
            gd.gd_launch_fenced(r.pool, 0, gd.GD_K_GEMM_BF16, gd.gd_args_gemm(Cc, A + size, B - 2 * size, M, N, K, 1), mode=gd.GD_FENCE_MODULO)
            r.sim.run("gemm_bf16", (base, size), ok.MODE_MODULO, Cc, A + size, B - 2 * size, M, N, K, 1, 0, M, 0, N)
            got, want = r.download(Cc, np.uint16, M * N), r.sim.view(Cc, np.uint16, M * N)
            assert_bf16_close(got, want, abs_tol=3e-5, what=f"modulo gemm {M}x{N}x{K}")
            # all three operands plainly inside, and all three one partition too high
            r.sim.run("gemm_bf16", (base, size), ok.MODE_MODULO, Cc, A, B, M, N, K, 1, 0, M, 0, N)
            want = r.sim.view(Cc, np.uint16, M * N).copy()
            plain = None
            for k in (0, 1):
                r.dev[Cc - r.base:Cc - r.base + 2 * M * N].fill_(0)
                gd.gd_launch_fenced(r.pool, 0, gd.GD_K_GEMM_BF16, gd.gd_args_gemm(Cc + k * size, A + k * size, B + k * size, M, N, K, 1), mode=gd.GD_FENCE_MODULO)
                got = r.download(Cc, np.uint16, M * N).copy()
                assert_bf16_close(got, want, abs_tol=3e-5, what=f"modulo gemm {M}x{N}x{K}, operands {k} partitions up")
                plain = got if plain is None else plain
                assert np.array_equal(got, plain), (M, N, K, k)
            r.dev[Cc - r.base:Cc - r.base + 2 * M * N].copy_(torch.from_numpy(want.view(np.uint8)))     # device = oracle again
        # nothing outside tenant 0's partition changed
        lo = r.table[1][0] - r.base
        assert np.all(r.dev[lo:].cpu().numpy() == 0xA5)
    finally:
        r.close()


# ---------------------------------------------------------------------------
# address checking
# ---------------------------------------------------------------------------

@pytest.fixture()
def checked():
    r = Rig([4 * MiB, 4 * MiB])
    counters = torch.zeros(8, dtype=torch.int64, device="cuda")
    gd.gd_pool_set_fault_counters(r.pool, counters.data_ptr(), 8)
    yield r, counters
    r.close()


def faults(counters, tenant):
    torch.cuda.synchronize()
    return int(counters[tenant].item())


def test_checking_stops_exactly_the_offending_threads_and_counts_them(checked):
    r, counters = checked
    (b0, s0), (b1, s1) = r.row(0), r.row(1)
    total = {0: 0, 1: 0}
    # stores that run over the end of partition 0, or start in front of partition 1
    for tenant, A, n in ((0, b0 + s0 - 4096, 5000), (1, b1 - 400, 300), (0, b0 + 64, 100), (1, b0, 50)):
        r.launch(tenant, gd.GD_K_STORE_TID, gd.gd_args_store_tid(A, n, 7 + tenant, 0), mode=gd.GD_FENCE_CHECK)
        r.oracle("store_tid", tenant, A, 7 + tenant, n, mode=ok.MODE_CHECK)
        total[tenant] += r.sim.last[1]
        assert faults(counters, tenant) == total[tenant]
        r.assert_images_equal(what="checked store_tid")
    assert total[0] == 5000 - 1024 and total[1] == 100 + 50

    # triad whose arrays straddle the end of the partition: vectors that cross are redone by element
    g = si.rng(6, 70)
    n = 40000
    for shift in (0, 4):
        a = b0 + s0 - 4 * 30000 + shift                  # last 10000 stores fall outside
        b, c = r.alloc(0, 4 * n + 64) + shift, r.alloc(0, 4 * n + 64) + (shift and 12)
        r.upload(0, b, si.uniform_f32(g, n))
        r.upload(0, c, si.uniform_f32(g, n))
        r.launch(0, gd.GD_K_TRIAD, gd.gd_args_triad(a, b, c, n, 0.5, 0), mode=gd.GD_FENCE_CHECK)
        r.oracle("triad", 0, a, b, c, 0.5, n, mode=ok.MODE_CHECK)
        assert r.sim.last[1] == 10000 + (1 if shift else 0)
        total[0] += r.sim.last[1]
        assert faults(counters, 0) == total[0]
        inb = 30000 - (1 if shift else 0)
        assert rel_frobenius(r.download(a, np.float32, inb), r.sim.view(a, np.float32, inb)) <= 1e-5
        r.assert_images_equal(skip=[(a, 4 * inb)], what="checked triad")
        r.launch(0, gd.GD_K_COPY, gd.gd_args_copy(b, c - 4 * n - 4 * MiB, n), mode=gd.GD_FENCE_CHECK)     # every load refused
        r.oracle("copy", 0, b, c - 4 * n - 4 * MiB, n, mode=ok.MODE_CHECK)
        total[0] += n
        assert r.sim.last[1] == n and faults(counters, 0) == total[0]
        r.assert_images_equal(skip=[(a, 4 * inb)], what="checked copy")


def test_checking_on_indexed_kernels_and_sum(checked):
    r, counters = checked
    t = 1
    base, size = r.row(t)
    g = si.rng(6, 80)
    n = 120003
    x, y, off, out = (r.alloc(t, 4 * n + 64) for _ in range(4))
    r.upload(t, x, si.uniform_f32(g, n))
    r.upload(t, y, si.uniform_f32(g, n))
    offs, where = si.c1_offsets(g, n, y, base, size, frac=0.02)
    r.upload(t, off, offs)
    total = 0
    r.launch(t, gd.GD_K_SAXPY_IDX, gd.gd_args_saxpy_idx(x, y, off, n, 0.25, 0), mode=gd.GD_FENCE_CHECK)
    r.oracle("saxpy_idx", t, x, y, off, 0.25, n, mode=ok.MODE_CHECK)
    total += r.sim.last[1]
    assert r.sim.last[1] == len(where) and faults(counters, t) == total
    assert rel_frobenius(r.download(y, np.float32, n), r.sim.view(y, np.float32, n)) <= 1e-5
    r.assert_images_equal(skip=[(y, 4 * n)], what="checked saxpy")
    # refused elements keep their old value bit for bit
    assert np.array_equal(r.download(y, np.uint32, n)[where], r.sim.view(y, np.uint32, n)[where])

    idx = r.alloc(t, 8 * n)
    ix, where = si.c2_indices(g, n, n, frac=0.01, oob_hi=1 << 34)
    ix[where[::2]] *= -1
    inside = (x + 4 * ix[where] >= base) & (x + 4 * ix[where] + 4 <= base + size)
    r.upload(t, idx, ix)
    r.dview(out, np.uint8, 4 * n).fill_(0x11)
    r.sim.view(out, np.uint8, 4 * n)[:] = 0x11
    r.launch(t, gd.GD_K_GATHER32_I64, gd.gd_args_gather(out, x, idx, n), mode=gd.GD_FENCE_CHECK)
    r.oracle("gather32_i64", t, out, x, idx, n, mode=ok.MODE_CHECK)
    total += r.sim.last[1]
    assert r.sim.last[1] == int((~inside).sum()) and faults(counters, t) == total
    racy = where[inside]                                  # in-partition but outside the table: may read `out`/`y`
    keep = np.ones(n, bool)
    keep[racy] = False
    assert np.array_equal(r.download(out, np.uint32, n)[keep], r.sim.view(out, np.uint32, n)[keep])
    assert np.all(r.download(out, np.uint32, n)[where[~inside]] == 0x11111111)

    r.launch(t, gd.GD_K_SCATTER_F32_I64, gd.gd_args_scatter(y, x, idx, n, 2.0, 0), mode=gd.GD_FENCE_CHECK)
    r.oracle("scatter_f32_i64", t, y, x, idx, 2.0, n, mode=ok.MODE_CHECK)
    total += r.sim.last[1]
    assert faults(counters, t) == total

    # sum over a range that runs past the end of the partition: the part inside is summed, the rest counted
    ws, res = r.alloc(t, gd.GD_SUM_WORKSPACE), r.alloc(t, 256)
    m = 50000
    start = base + size - 4 * 30000
    r.upload(t, start, si.uniform_f32(g, 30000, 0.0, 1.0))
    r.launch(t, gd.GD_K_SUM_F32, gd.gd_args_sum(res, start, ws, m), mode=gd.GD_FENCE_CHECK)
    exact = r.oracle("sum_f32_exact", t, start, m, mode=ok.MODE_CHECK)
    assert r.sim.last[1] == 20000
    total += 20000
    assert faults(counters, t) == total
    assert abs(float(r.download(res, np.float32, 1)[0]) - exact) <= 1e-5 * exact
    assert faults(counters, 0) == 0


def test_checking_rmsnorm_stops_rows_and_elements_and_counts_them(checked):
    """Thread (r, j) reads all of row r, then g[j], then stores y[r,j] (Sections 4.3, 4.4): a row of x
    that is not wholly inside stops all of its threads, a gain or an output outside stops one thread."""
    r, counters = checked
    t = 0
    base, size = r.row(t)
    end = base + size
    g = si.rng(6, 90)
    total = 0
    for rows, cols, shift in ((12, 2048, 0), (5, 8192, 0), (9, 1000, 0), (7, 520, 2)):
        nbytes = 2 * rows * cols
        xin = r.alloc(t, nbytes + 64) + shift
        gain_in = r.alloc(t, 2 * cols + 64) + shift
        yin = r.alloc(t, nbytes + 64) + shift
        r.upload(t, xin, si.f32_to_bf16_bits(si.normal_f32(g, rows * cols)))
        r.upload(t, gain_in, si.f32_to_bf16_bits(si.uniform_f32(g, cols, 0.5, 1.5)))
        # the last bytes of the partition: free of allocations in this rig (4 MiB, a few hundred KiB in use)
        r.upload(t, end - 2 * cols, si.f32_to_bf16_bits(si.uniform_f32(g, cols, 0.5, 1.5)))
        r.upload(t, end - 4 * cols - nbytes, si.f32_to_bf16_bits(si.normal_f32(g, rows * cols + cols)))
        cases = [
            (yin, xin, gain_in),                                         # everything inside
            (yin, xin, end - 2 * (cols - 37)),                           # the last 37 gains are outside
            (yin, end - nbytes + 2 * (cols // 3), gain_in),              # the last third of x's last row is outside
            (end - nbytes + 2 * (2 * cols + 21), xin, gain_in),          # y leaves the partition in row rows-3
            (yin, base - 2 * (cols + 5), gain_in),                       # x starts in front: rows 0 and 1 are refused
        ]
        for (y, x, gain) in cases:
            r.dview(yin - shift, np.uint8, nbytes + 64).fill_(0x33)
            r.sim.view(yin - shift, np.uint8, nbytes + 64)[:] = 0x33
            r.launch(t, gd.GD_K_RMSNORM_BF16, gd.gd_args_rmsnorm(y, x, gain, rows, cols, 1e-6, 0), mode=gd.GD_FENCE_CHECK)
            r.oracle("rmsnorm_bf16", t, y, x, gain, rows, cols, 1e-6, mode=ok.MODE_CHECK)
            total += r.sim.last[1]
            assert faults(counters, t) == total, (rows, cols, shift, hex(y), hex(x), hex(gain), r.sim.last)
            got, want = r.image(), r.sim.mem
            # bf16 outputs may differ by a unit in the last place; every byte the oracle left alone is left alone
            changed = got != want
            if changed.any():
                pos = np.flatnonzero(changed) // 2 * 2
                pos = np.unique(pos)
                gb = got[pos].astype(np.uint16) | (got[pos + 1].astype(np.uint16) << 8)
                wb = want[pos].astype(np.uint16) | (want[pos + 1].astype(np.uint16) << 8)
                assert_bf16_close(gb, wb, flip_budget=1.0, frobenius=False, what="checked rmsnorm")
                assert pos.size <= 0.02 * rows * cols + 2
            # same bits on both sides again before the next case reads what this one wrote
            r.dview(base, np.uint8, size).copy_(torch.from_numpy(r.sim.view(base, np.uint8, size)))
        assert total > 0
        for p in (xin - shift, gain_in - shift, yin - shift):
            r.free(t, p)
    assert faults(counters, 1) == 0


def test_checking_gemm_stops_threads_with_a_refused_operand_row_or_column(checked):
    """Thread (m, n) needs row m of A, column n of B and C[m,n]; tile-multiple, ragged and generic shapes."""
    r, counters = checked
    t = 1
    base, size = r.row(t)
    end = base + size
    g = si.rng(6, 91)
    total = 0
    for (M, N, K, b_is_nk) in ((256, 256, 128, 1), (512, 256, 384, 1), (256, 256, 320, 1), (300, 200, 72, 1), (64, 40, 24, 0), (50, 70, 33, 1)):
        A_in, B_in, C_in = r.alloc(t, 2 * M * K), r.alloc(t, 2 * K * N), r.alloc(t, 2 * M * N)
        a_bits = si.f32_to_bf16_bits(si.normal_f32(g, M * K) * np.float32(K ** -0.5))
        b_bits = si.f32_to_bf16_bits(si.normal_f32(g, K * N))
        r.upload(t, A_in, a_bits)
        r.upload(t, B_in, b_bits)
        # a copy of A that runs over the end of the partition
        a_cut = 2 * (K * (M - M // 3) + 16)
        r.upload(t, end - a_cut, a_bits[: a_cut // 2])
        A_over = end - a_cut                                            # rows from about 2M/3 on are not wholly inside
        cases = [(C_in, A_in, B_in),
                 (C_in, A_over, B_in),
                 (end - 2 * (N * (M // 2) + N // 4), A_in, B_in),       # C leaves the partition in its middle row
                 (C_in, A_in, base - 2 * (3 * K + 8) if b_is_nk else base - 2 * 5)]   # B starts in front of the partition
        for (Cc, A, B) in cases:
            r.dview(C_in, np.uint8, 2 * M * N).fill_(0x33)
            r.sim.view(C_in, np.uint8, 2 * M * N)[:] = 0x33
            r.launch(t, gd.GD_K_GEMM_BF16, gd.gd_args_gemm(Cc, A, B, M, N, K, b_is_nk), mode=gd.GD_FENCE_CHECK)
            r.oracle("gemm_bf16", t, Cc, A, B, M, N, K, b_is_nk, 0, M, 0, N, mode=ok.MODE_CHECK)
            total += r.sim.last[1]
            assert faults(counters, t) == total, (M, N, K, b_is_nk, hex(Cc), hex(A), hex(B), r.sim.last)
            got, want = r.image(), r.sim.mem
            changed = got != want
            if changed.any():
                pos = np.unique(np.flatnonzero(changed) // 2 * 2)
                gb = got[pos].astype(np.uint16) | (got[pos + 1].astype(np.uint16) << 8)
                wb = want[pos].astype(np.uint16) | (want[pos + 1].astype(np.uint16) << 8)
                assert_bf16_close(gb, wb, abs_tol=3e-5, flip_budget=1.0, frobenius=False, what="checked gemm")
                assert pos.size <= 0.02 * M * N + 2
            r.dview(base, np.uint8, size).copy_(torch.from_numpy(r.sim.view(base, np.uint8, size)))
        for p in (A_in, B_in, C_in):
            r.free(t, p)
    assert total > 0 and faults(counters, 0) == 0


# ---------------------------------------------------------------------------
# address checking by the memory pipeline (buffer instructions)
# ---------------------------------------------------------------------------

def images_close_bf16(r, what, budget):
    """Whole pool image against the oracle's: bytes equal, except bf16 outputs that differ by one unit."""
    torch.cuda.synchronize()
    got, want = r.dev.cpu().numpy(), r.sim.mem
    changed = got != want
    if changed.any():
        pos = np.unique(np.flatnonzero(changed) // 2 * 2)
        gb = got[pos].astype(np.uint16) | (got[pos + 1].astype(np.uint16) << 8)
        wb = want[pos].astype(np.uint16) | (want[pos + 1].astype(np.uint16) << 8)
        assert_bf16_close(gb, wb, abs_tol=3e-5, flip_budget=1.0, frobenius=False, what=what)
        assert pos.size <= budget, (what, pos.size)


def test_pointer_chase_in_every_rule_ends_where_the_oracle_ends():
    """The dependent chain behind the latency figures: last indices equal the oracle's bit for bit in every rule,
    also when the walk meets entries that point outside the partition (wrapped, zero, or the thread stops and
    is counted); the two counters are measurements and only have to be plausible."""
    r = Rig([4 * MiB, 4 * MiB])
    counters = torch.zeros(8, dtype=torch.int64, device="cuda")
    gd.gd_pool_set_fault_counters(r.pool, counters.data_ptr(), 8)
    try:
        g = si.rng(7, 2)
        t = 1
        base, size = r.row(t)
        tab_host, first = si.chase_table(g, MiB)
        tab, out, clk = r.alloc(t, tab_host.nbytes), r.alloc(t, 256), r.alloc(t, 256)
        total = 0
        modes = ((gd.GD_FENCE_BITWISE, ok.MODE_BITWISE), (gd.GD_FENCE_MODULO, ok.MODE_MODULO), (gd.GD_FENCE_CHECK, ok.MODE_CHECK),
                 (gd.GD_FENCE_HWCHECK, ok.MODE_HWCHECK), (gd.GD_FENCE_NONE, ok.MODE_NONE))
        for planted in (False, True):
            host = tab_host.copy()
            if planted:
                # every 7th line in use points somewhere outside: far beyond, just behind the end, in front of the start
                used = np.arange(0, host.size, 32)[::7]
                host[used] = np.where(np.arange(used.size) % 3 == 0, np.uint32(0xFFFFFF00),
                                      np.where(np.arange(used.size) % 3 == 1, np.uint32((base + size - tab) // 4 + 5), np.uint32(2**32 - 40)))
            r.upload(t, tab, host)
            for mode, omode in modes:
                if planted and mode == gd.GD_FENCE_NONE:
                    continue                                     # the unfenced kernel only ever sees in-bounds walks
                # every start is a line in use (entry 0 is one, and so is every 32nd), so that an unfenced walk stays inside
                for steps, threads, hop, start in ((1000, 1, 0, first), (333, 64, 32, 0), (0, 3, 1, 0)):
                    for ptr, fill in ((out, 0x11), (clk, 0)):
                        r.dview(ptr, np.uint8, 256).fill_(fill)
                        r.sim.view(ptr, np.uint8, 256)[:] = fill
                    r.launch(t, gd.GD_K_CHASE, gd.gd_args_chase(out, clk, tab, steps, start, hop, threads, 0), mode=mode)
                    r.oracle("chase", t, out, clk, tab, steps, start, hop, threads, mode=omode)
                    if mode == gd.GD_FENCE_CHECK:
                        total += r.sim.last[1]
                        assert faults(counters, t) == total
                    if planted and steps:
                        assert r.sim.last[1] + r.sim.last[2] > 0
                    r.assert_images_equal(skip=[(clk, 16)], what=f"chase mode {mode} steps {steps} threads {threads}")
                    cycles, ticks = (int(v) for v in r.download(clk, np.uint64, 2))
                    if steps == 1000 and not planted:
                        # a dependent load cannot take under 20 cycles, nor a microsecond; 100 MHz ticks against cycles: 0.5 .. 3 GHz
                        assert 20 * steps < cycles < 100000 * steps and 5 * ticks < cycles < 40 * ticks + 2000, (cycles, ticks)
        assert total > 0
        with pytest.raises(gd.GuardianError):
            r.launch(t, gd.GD_K_CHASE, gd.gd_args_chase(out, clk, tab, 1, first, 0, 65, 0))
        with pytest.raises(gd.GuardianError):
            r.launch(t, gd.GD_K_CHASE, gd.gd_args_chase(out, clk, tab, 1, first, 0, 1, 0), grid=(2, 1, 1))
    finally:
        r.close()


def test_rmsnorm_of_many_rows_in_every_rule():
    """Matrices of a few thousand rows (more workgroups than the chip holds at once) with 4096 or 8192 columns,
    in every rule, against the oracle: whole pool image, bf16 results within a unit, exact fault counts; through
    pointers the rule maps back, with the output leaving the partition and the input starting in front of it."""
    r = Rig([128 * MiB, 4 * MiB])
    counters = torch.zeros(8, dtype=torch.int64, device="cuda")
    gd.gd_pool_set_fault_counters(r.pool, counters.data_ptr(), 8)
    try:
        g = si.rng(6, 97)
        t = 0
        base, size = r.row(t)
        end = base + size
        total = 0
        for rows, cols in ((2050, 8192), (2049, 4096), (3077, 4096)):
            nbytes = 2 * rows * cols
            pad = r.alloc(t, 64 * KiB)                # where stores that wrap under the bitwise rule land: nothing reads it
            x, y, gain = r.alloc(t, nbytes), r.alloc(t, nbytes), r.alloc(t, 2 * cols)
            r.upload(t, x, si.f32_to_bf16_bits(si.normal_f32(g, rows * cols)))
            r.upload(t, gain, si.f32_to_bf16_bits(si.uniform_f32(g, cols, 0.5, 1.5)))
            args = gd.gd_args_rmsnorm(y, x, gain, rows, cols, 1e-6, 0)
            # every rule on plain operands, and the unfenced kernel bit for bit equal to the bitwise rule
            r.oracle("rmsnorm_bf16", t, y, x, gain, rows, cols, 1e-6)
            first = None
            for mode in (gd.GD_FENCE_BITWISE, gd.GD_FENCE_MODULO, gd.GD_FENCE_CHECK, gd.GD_FENCE_HWCHECK, gd.GD_FENCE_NONE):
                r.dview(y, np.uint8, nbytes).fill_(0x33)
                r.launch(t, gd.GD_K_RMSNORM_BF16, args, mode=mode)
                images_close_bf16(r, f"rmsnorm {rows}x{cols} mode {mode}", 0.02 * rows * cols + 2)
                got = r.download(y, np.uint16, rows * cols)
                first = got if first is None else first
                assert np.array_equal(got, first), mode
            assert faults(counters, t) == total
            # pointers that the rule maps back: one partition too high or too low (bitwise and modulo)
            for mode, omode in ((gd.GD_FENCE_BITWISE, ok.MODE_BITWISE), (gd.GD_FENCE_MODULO, ok.MODE_MODULO)):
                r.dview(y, np.uint8, nbytes).fill_(0x33)
                r.launch(t, gd.GD_K_RMSNORM_BF16, gd.gd_args_rmsnorm(y + size, x - size, gain + 3 * size, rows, cols, 1e-6, 0), mode=mode)
                assert np.array_equal(r.download(y, np.uint16, rows * cols), first), mode
            if cols == 8192:
                # the output leaves the partition in its last rows: address checking refuses those threads, the
                # hardware-checked rule drops their stores, the bitwise rule wraps them to the partition's start
                hang = 2 * (2 * cols + 24)
                y_end = end - nbytes + hang
                for mode, omode in ((gd.GD_FENCE_CHECK, ok.MODE_CHECK), (gd.GD_FENCE_HWCHECK, ok.MODE_HWCHECK), (gd.GD_FENCE_BITWISE, ok.MODE_BITWISE)):
                    r.launch(t, gd.GD_K_RMSNORM_BF16, gd.gd_args_rmsnorm(y_end, x, gain, rows, cols, 1e-6, 0), mode=mode)
                    r.oracle("rmsnorm_bf16", t, y_end, x, gain, rows, cols, 1e-6, mode=omode)
                    assert r.sim.last[2 if mode == gd.GD_FENCE_BITWISE else 1] == hang // 2       # wrapped, resp. refused
                    if mode == gd.GD_FENCE_CHECK:
                        total += r.sim.last[1]
                        assert faults(counters, t) == total
                    images_close_bf16(r, f"rmsnorm over the end, mode {mode}", 0.02 * rows * cols + 2)
                    r.dview(base, np.uint8, size).copy_(torch.from_numpy(r.sim.view(base, np.uint8, size)))
                # the input starts in front of the partition: the hardware-checked rule reads zeros there
                x_front = base - 2 * (cols + 40)
                r.launch(t, gd.GD_K_RMSNORM_BF16, gd.gd_args_rmsnorm(y, x_front, gain, rows, cols, 1e-6, 0), mode=gd.GD_FENCE_HWCHECK)
                r.oracle("rmsnorm_bf16", t, y, x_front, gain, rows, cols, 1e-6, mode=ok.MODE_HWCHECK)
                assert r.sim.last[1] > 0
                images_close_bf16(r, "rmsnorm from in front, hardware checked", 0.02 * rows * cols + 2)
            for ptr in (pad, x, y, gain):
                r.free(t, ptr)
            r.dview(base, np.uint8, size).copy_(torch.from_numpy(r.sim.view(base, np.uint8, size)))
    finally:
        r.close()


def test_hwcheck_on_odd_sized_partitions_matches_the_oracle():
    sizes = [3 * MiB + 256, 5 * MiB + 768, MiB + 256 * 17]
    r = FlexRig(sizes)
    try:
        g = si.rng(6, 95)
        mode, omode = gd.GD_FENCE_HWCHECK, ok.MODE_HWCHECK
        for t, (base, size) in enumerate(r.table):
            end = base + size
            n = 20001
            raw = random_addresses(g, n, base, size)
            raw[n // 2: n // 2 + 2000] = np.uint64(base) + g.integers(0, size, size=2000, dtype=np.uint64) + np.uint64(3 << 32)
            src, dst = r.alloc(t, 8 * n), r.alloc(t, 8 * n)
            r.upload(t, src, raw)
            for width in (1, 2, 4, 8, 16):
                gd.gd_launch_fenced(r.pool, t, gd.GD_K_FENCE_ADDRS, gd.gd_args_fence_addrs(dst, src, n, width, 0), mode=mode)
                r.sim.run("fence_addrs", (base, size), omode, dst, src, width, n)
                got = r.download(dst, np.uint64, n)
                want = ok.fence_array(base, size, raw, width, omode)
                assert np.array_equal(got, want)
                made = got != np.uint64(hm.U64)
                assert made.any() and (~made).any()
                assert got[made].min() >= base and got[made].max() + width <= end
            # a store loop that starts in front of the partition and runs past its end: only the part inside is written
            gd.gd_launch_fenced(r.pool, t, gd.GD_K_STORE_TID, gd.gd_args_store_tid(base - 1000 * 4, size // 4 + 3000, 40 + t, 0), mode=mode)
            r.sim.run("store_tid", (base, size), omode, base - 1000 * 4, 40 + t, size // 4 + 3000)
            assert r.sim.last[1] == 3000 and r.images_equal(), f"tenant {t}"
        t = 1
        base, size = r.table[t]
        end = base + size
        n = 100003
        r.upload(t, base, si.uniform_f32(g, 50003))
        for shift in (0, 4):                                     # 16-byte aligned: the tile path; misaligned: per element
            a = end - 4 * 30000 + shift                          # the last 70003 stores fall outside
            b = base + 512 * KiB + shift
            c = base - 4 * 50000 + (shift and 12)                # the first 50000 loads of c lie in front of the partition: they read 0
            r.upload(t, b, si.uniform_f32(g, n))
            gd.gd_launch_fenced(r.pool, t, gd.GD_K_TRIAD, gd.gd_args_triad(a, b, c, n, 0.75, 0), mode=mode)
            r.sim.run("triad", (base, size), omode, a, b, c, 0.75, n)
            inb = 30000 - (1 if shift else 0)
            assert r.sim.last[1] == (n - inb) + (50000 - (3 if shift else 0))
            assert rel_frobenius(r.download(a, np.float32, inb), r.sim.view(a, np.float32, inb)) <= 1e-5
            assert r.images_equal(skip=[(a, 4 * inb)])
            r.upload(t, a, r.sim.view(a, np.float32, inb).copy())
            gd.gd_launch_fenced(r.pool, t, gd.GD_K_COPY, gd.gd_args_copy(base + 2 * MiB + shift, a, n), mode=mode)
            r.sim.run("copy", (base, size), omode, base + 2 * MiB + shift, a, n)
            assert r.images_equal()
        # gather with indices far outside (offsets wrap at 2^32: some land inside, most are refused)
        tab, idx, out = base + 512 * KiB, base + MiB, base + 2 * MiB
        m = 60001
        ix, where = si.c2_indices(g, m, 100000, frac=0.02, oob_hi=1 << 40)
        ix[where[::3]] *= -1
        img = ok.fence_array(base, size, np.uint64(tab) + (4 * ix[where]).astype(np.uint64), 4, omode)
        ix[where[(img >= out) & (img < out + 4 * m)]] = 5         # loads that would race with this launch's stores
        r.upload(t, idx, ix)
        gd.gd_launch_fenced(r.pool, t, gd.GD_K_GATHER32_I64, gd.gd_args_gather(out, tab, idx, m), mode=mode)
        r.sim.run("gather32_i64", (base, size), omode, out, tab, idx, m)
        assert r.sim.last[1] > 0.9 * len(where) and r.images_equal()
        # scatter: indices outside are refused (offsets far beyond the size); duplicates may land in either order
        ix2 = g.integers(0, 100000, size=m, dtype=np.int64)
        ix2[::50] = (1 << 28) + np.arange(len(ix2[::50]))
        ix2[7::50] = -(1 << 20) - np.arange(len(ix2[7::50]))
        r.upload(t, idx, ix2)
        dst = base + 3 * MiB
        gd.gd_launch_fenced(r.pool, t, gd.GD_K_SCATTER_F32_I64, gd.gd_args_scatter(dst, out, idx, m, 2.0, 0), mode=mode)
        r.sim.run("scatter_f32_i64", (base, size), omode, dst, out, idx, 2.0, m)
        assert r.sim.last[1] == len(ix2[::50]) + len(ix2[7::50])
        assert r.images_equal(skip=[(dst, 4 * 100000)])
        inr = ix2[(ix2 >= 0) & (ix2 < 100000)]
        once = np.flatnonzero(np.bincount(inr, minlength=100000) <= 1)
        assert np.array_equal(r.download(dst, np.uint32, 100000)[once], r.sim.view(dst, np.uint32, 100000)[once])
        ws, res = base + 4 * MiB, base + 4 * MiB + 64 * KiB
        start = end - 4 * 30000
        gd.gd_launch_fenced(r.pool, t, gd.GD_K_SUM_F32, gd.gd_args_sum(res, start, ws, 50000), mode=mode)
        exact = r.sim.run("sum_f32_exact", (base, size), omode, start, 50000)
        assert r.sim.last[1] == 20000
        assert abs(float(r.download(res, np.float32, 1)[0]) - exact) <= 1e-5 * abs(exact)
        # the neighbours never changed
        for other in (0, 2):
            ob, os_ = r.table[other]
            assert np.array_equal(r.download(ob, np.uint8, os_), r.sim.view(ob, np.uint8, os_))
    finally:
        r.close()


def test_hwcheck_rmsnorm_and_gemm_read_zero_outside_and_drop_stores():
    r = Rig([4 * MiB, 4 * MiB])
    try:
        g = si.rng(6, 96)
        mode, omode = gd.GD_FENCE_HWCHECK, ok.MODE_HWCHECK
        t = 0
        base, size = r.row(t)
        end = base + size
        rows, cols = 9, 2048
        x, gain = r.alloc(t, 2 * rows * cols), r.alloc(t, 2 * cols)
        r.upload(t, x, si.f32_to_bf16_bits(si.normal_f32(g, rows * cols)))
        r.upload(t, gain, si.f32_to_bf16_bits(si.uniform_f32(g, cols, 0.5, 1.5)))
        r.upload(t, end - 2 * rows * cols, si.f32_to_bf16_bits(si.normal_f32(g, rows * cols)))
        for (y, xx) in ((end - 2 * (6 * cols + 104), x),                    # output leaves the partition in row 6 (16-byte aligned)
                        (base + 2 * MiB, end - 2 * rows * cols + 2 * (cols + 304)),    # input: the end of the last rows reads zeros
                        (base + 2 * MiB + 2, end - 2 * rows * cols + 2 * 77),         # the same through pointers that are not 16-byte aligned
                        (end - 2 * (3 * cols + 101), x + 2)):
            gd.gd_launch_fenced(r.pool, t, gd.GD_K_RMSNORM_BF16, gd.gd_args_rmsnorm(y, xx, gain, rows, cols, 1e-6, 0), mode=mode)
            r.oracle("rmsnorm_bf16", t, y, xx, gain, rows, cols, 1e-6, mode=omode)
            assert r.sim.last[1] > 0
            images_close_bf16(r, "hwcheck rmsnorm", 0.02 * rows * cols + 2)
            r.dview(base, np.uint8, size).copy_(torch.from_numpy(r.sim.view(base, np.uint8, size)))
        for (M, N, K, b_is_nk) in ((256, 256, 128, 1), (512, 256, 384, 1), (256, 256, 320, 1), (300, 200, 72, 1), (50, 70, 33, 0)):
            A, B, Cc = r.alloc(t, 2 * M * K), r.alloc(t, 2 * K * N), r.alloc(t, 2 * M * N)
            a_bits = si.f32_to_bf16_bits(si.normal_f32(g, M * K) * np.float32(K ** -0.5))
            r.upload(t, A, a_bits)
            r.upload(t, B, si.f32_to_bf16_bits(si.normal_f32(g, K * N)))
            a_cut = 2 * (K * (M - M // 3) + 16)
            r.upload(t, end - a_cut, a_bits[: a_cut // 2])
            cases = [(Cc, A, B), (Cc, end - a_cut, B), (end - 2 * (N * (M // 2) + N // 4), A, B)]
            if (2 * K) % 128 == 0:
                # the same cut at a whole row, so that the pointer keeps the 128-byte alignment of the DMA-ring kernel:
                # its buffer loads to the LDS deliver zeros for the rows behind the partition's end
                cases.append((Cc, end - 2 * K * (M - M // 3), B))
            for (cc, aa, bb) in cases:
                gd.gd_launch_fenced(r.pool, t, gd.GD_K_GEMM_BF16, gd.gd_args_gemm(cc, aa, bb, M, N, K, b_is_nk), mode=mode)
                r.oracle("gemm_bf16", t, cc, aa, bb, M, N, K, b_is_nk, 0, M, 0, N, mode=omode)
                images_close_bf16(r, f"hwcheck gemm {M}x{N}x{K}", 0.02 * M * N + 2)
                r.dview(base, np.uint8, size).copy_(torch.from_numpy(r.sim.view(base, np.uint8, size)))
            for p in (A, B, Cc):
                r.free(t, p)
        b1, s1 = r.row(1)
        assert np.all(r.download(b1, np.uint8, s1) == 0xA5)
    finally:
        r.close()
