"""GPU parity: every kernel of the library, launched through the C ABI, against
the CPU oracle on the same seeded inputs at the same device addresses.

Bars.  Integer, byte and index results and the whole memory image outside
floating-point outputs: bit-exact.  fp32 outputs: relative Frobenius error
<= 1e-5 against the oracle's fp64 arithmetic.  bf16 outputs: <= 1e-3 against the
oracle's result rounded to bf16.  Fenced output is bit-identical to unfenced
output on in-bounds inputs.
"""
import numpy as np
import pytest
import torch

import paper_2401_09290_amd as gd
import synth_inputs as si
from harness import GiB, KiB, MiB, Rig, assert_bf16_close, rel_frobenius
from oracle import kernels as ok

pytestmark = pytest.mark.gpu

FP32_TOL = 1e-5
BF16_TOL = 1e-3
# fp32 accumulation of K products of magnitude ~1/sqrt(K) each (entries of C ~ N(0,1)): a few 1e-6
# absolute for K up to 8192; it decides the bf16 rounding only for entries that close to zero.
GEMM_ABS_TOL = 3e-5


@pytest.fixture()
def rig2():
    r = Rig([4 * MiB, 4 * MiB])
    yield r
    r.close()


# ---------------------------------------------------------------------------
# Listing 1's kernel and the fence probe
# ---------------------------------------------------------------------------

def test_store_tid_in_bounds_overrun_and_foreign_pointer(rig2):
    r = rig2
    (b0, s0), (b1, s1) = r.row(0), r.row(1)
    cases = [(0, b0 + 4096, 7, 1000),                 # in bounds
             (0, b0 + s0 - 4096, 8, 5000),            # runs over the end of partition 0: wraps to its start
             (1, b0 + 64, 9, 777),                    # tenant 1 passes a pointer into partition 0
             (1, b1 - 4 * 100, 10, 300),              # starts in front of its partition
             (0, b0 + 2, 11, 5),                      # misaligned pointer: low bits dropped
             (1, (1 << 64) - 8192 + 4, 13, 5000),     # a pointer just below 2^64: the element addresses wrap through zero
             (0, 0, 14, 3000),                        # the null pointer
             (0, b0, 12, 0)]                          # empty launch
    for tenant, A, j, n in cases:
        r.launch(tenant, gd.GD_K_STORE_TID, gd.gd_args_store_tid(A, n, j, 0))
        r.oracle("store_tid", tenant, A, j, n)
        r.assert_images_equal(what=f"store_tid tenant {tenant} A={A:#x} n={n}")


@pytest.mark.parametrize("width", [1, 2, 4, 8, 16])
def test_fence_probe_matches_oracle_bit_exactly(rig2, width):
    r = rig2
    g = si.rng(0, 10 + width)
    for tenant in (0, 1):
        base, size = r.row(tenant)
        n = 40001
        raw = g.integers(0, 1 << 63, size=n, dtype=np.uint64) * np.uint64(2) + g.integers(0, 2, size=n, dtype=np.uint64)
        near = (np.uint64(base) + g.integers(0, 4 * size, size=n // 2, dtype=np.uint64) - np.uint64(2 * size))
        raw[: n // 2] = near
        src, dst = r.alloc(tenant, 8 * n), r.alloc(tenant, 8 * n)
        r.upload(tenant, src, raw)
        r.launch(tenant, gd.GD_K_FENCE_ADDRS, gd.gd_args_fence_addrs(dst, src, n, width, 0))
        r.oracle("fence_addrs", tenant, dst, src, width, n)
        got = r.download(dst, np.uint64, n)
        assert np.array_equal(got, ok.fence_array(base, size, raw, width))
        assert got.min() >= base and got.max() + width <= base + size
        r.assert_images_equal(what="fence probe")
        # protection off: the probe reports the raw addresses
        r.launch(tenant, gd.GD_K_FENCE_ADDRS, gd.gd_args_fence_addrs(dst, src, n, width, 0), mode=gd.GD_FENCE_NONE)
        assert np.array_equal(r.download(dst, np.uint64, n), raw)
        r.oracle("fence_addrs", tenant, dst, src, width, n, mode=ok.MODE_NONE)


def test_fence_probe_on_a_partition_larger_than_4gib():
    r = Rig([8 * GiB], fill=None, simulate=False)
    try:
        base, size = r.row(0)
        g = si.rng(0, 30)
        n = 100000
        raw = g.integers(0, 1 << 63, size=n, dtype=np.uint64) * np.uint64(2) + g.integers(0, 2, size=n, dtype=np.uint64)
        raw[: n // 2] = np.uint64(base) + g.integers(0, 4 * size, size=n // 2, dtype=np.uint64) - np.uint64(2 * size)
        # the probe's own arrays sit above the 4 GiB line of the partition
        r.alloc(0, 5 * GiB)
        src, dst = r.alloc(0, 8 * n), r.alloc(0, 8 * n)
        assert src - base > 4 * GiB
        r.upload(0, src, raw)
        for width in (1, 4, 16):
            r.launch(0, gd.GD_K_FENCE_ADDRS, gd.gd_args_fence_addrs(dst, src, n, width, 0))
            got = r.download(dst, np.uint64, n)
            assert np.array_equal(got, ok.fence_array(base, size, raw, width))
        # wrapped pointers: the same launch through aliases one partition size away
        r.dview(dst, np.uint64, n).zero_()
        r.launch(0, gd.GD_K_FENCE_ADDRS, gd.gd_args_fence_addrs(dst + size, src - size, n, 8, 0))
        assert np.array_equal(r.download(dst, np.uint64, n), ok.fence_array(base, size, raw, 8))
    finally:
        r.close()


# ---------------------------------------------------------------------------
# copy / triad
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("n,shift", [(0, 0), (1, 0), (3, 0), (1023, 0), (4096, 0), (100003, 0), (262144 + 5, 0),
                                     (100003, 4), (5000, 8)])
def test_copy_and_triad_against_oracle_and_unfenced(rig2, n, shift):
    r = rig2
    g = si.rng(0, 40)
    a = r.alloc(0, 4 * n + 64) + shift          # shift: pointers that are not 16-byte aligned
    b = r.alloc(0, 4 * n + 64) + shift
    c = r.alloc(0, 4 * n + 64) + (shift and 12)
    vb, vc = si.uniform_f32(g, n), si.uniform_f32(g, n)
    r.upload(0, b, vb)
    r.upload(0, c, vc)
    s = float(np.float32(0.7391))
    for kid, args, oname, oargs in (
            (gd.GD_K_COPY, gd.gd_args_copy(a, b, n), "copy", (a, b, n)),
            (gd.GD_K_TRIAD, gd.gd_args_triad(a, b, c, n, s, 0), "triad", (a, b, c, s, n))):
        r.launch(0, kid, args)
        r.oracle(oname, 0, *oargs)
        fenced = r.download(a, np.float32, n)
        want = r.sim.view(a, np.float32, n)
        if oname == "copy":
            assert np.array_equal(fenced.view(np.uint32), want.view(np.uint32))
            r.assert_images_equal(what=f"copy n={n}")
        else:
            assert rel_frobenius(fenced, want) <= FP32_TOL
            r.assert_images_equal(skip=[(a, 4 * n)], what=f"triad n={n}")
        r.dview(a, np.uint8, 4 * n).fill_(0)
        r.launch(0, kid, args, mode=gd.GD_FENCE_NONE)
        assert np.array_equal(r.download(a, np.float32, n).view(np.uint32), fenced.view(np.uint32))


def test_triad_caller_chosen_launch_shapes(rig2):
    r = rig2
    n = 70001
    g = si.rng(0, 41)
    a, b, c = (r.alloc(0, 4 * n) for _ in range(3))
    r.upload(0, b, si.uniform_f32(g, n))
    r.upload(0, c, si.uniform_f32(g, n))
    r.oracle("triad", 0, a, b, c, 0.25, n)
    want = r.sim.view(a, np.float32, n).copy()
    for grid, block in (((1, 1, 1), (64, 1, 1)), ((7, 1, 1), (1024, 1, 1)), ((1000, 1, 1), (128, 1, 1))):
        r.dview(a, np.uint8, 4 * n).fill_(0)
        r.launch(0, gd.GD_K_TRIAD, gd.gd_args_triad(a, b, c, n, 0.25, 0), grid=grid, block=block)
        assert rel_frobenius(r.download(a, np.float32, n), want) <= FP32_TOL
    for grid, block in (((0, 1, 1), (64, 1, 1)), ((1, 1, 1), (96, 1, 1)), ((1, 1, 1), (2048, 1, 1)), ((1, 2, 1), (64, 1, 1))):
        with pytest.raises(gd.GuardianError) as e:
            r.launch(0, gd.GD_K_TRIAD, gd.gd_args_triad(a, b, c, n, 0.25, 0), grid=grid, block=block)
        assert e.value.status == gd.GD_EINVAL


def test_triad_through_out_of_partition_pointers_wraps_into_own_partition(rig2):
    # Tenant 1 passes pointers that lie in tenant 0's partition: its kernel reads
    # and writes the same offsets of its own partition instead.
    r = rig2
    (b0, s0), (b1, s1) = r.row(0), r.row(1)
    n = 50000
    g = si.rng(0, 42)
    for t in (0, 1):
        for k in range(3):
            p = r.alloc(t, 4 * n)
            r.upload(t, p, si.uniform_f32(g, n))
    a0, bb0, c0 = b0, b0 + 4 * n + (-4 * n) % 256, b0 + 2 * (4 * n + (-4 * n) % 256)
    r.launch(1, gd.GD_K_TRIAD, gd.gd_args_triad(a0, bb0, c0, n, 1.5, 0))
    r.oracle("triad", 1, a0, bb0, c0, 1.5, n)
    a1 = a0 - b0 + b1
    assert rel_frobenius(r.download(a1, np.float32, n), r.sim.view(a1, np.float32, n)) <= FP32_TOL
    r.assert_images_equal(skip=[(a1, 4 * n)], what="foreign-pointer triad")


@pytest.mark.parametrize("repeat", [2, 7])
@pytest.mark.parametrize("mode", [gd.GD_FENCE_NONE, gd.GD_FENCE_BITWISE, gd.GD_FENCE_MODULO, gd.GD_FENCE_CHECK])
def test_triad_repeat_field_gives_the_single_pass_image(mode, repeat):
    """The triad's `repeat` field performs the same pass several times inside one launch (the
    cache-resident regime the benchmark times); the image must be that of one pass, in every
    fence variant, for aligned and misaligned pointers and for caller-chosen launch shapes."""
    r = Rig([4 * MiB, 4 * MiB])
    try:
        counters = torch.zeros(4, dtype=torch.int64, device="cuda")
        gd.gd_pool_set_fault_counters(r.pool, counters.data_ptr(), 4)
        omode = {gd.GD_FENCE_NONE: ok.MODE_NONE, gd.GD_FENCE_BITWISE: ok.MODE_BITWISE,
                 gd.GD_FENCE_MODULO: ok.MODE_MODULO, gd.GD_FENCE_CHECK: ok.MODE_CHECK}[mode]
        g = si.rng(0, 43)
        for n, shift, shape in ((100003, 0, {}), (30001, 4, {}), (65536, 0, dict(grid=(3, 1, 1), block=(256, 1, 1)))):
            a = r.alloc(0, 4 * n + 64) + shift
            b = r.alloc(0, 4 * n + 64) + shift
            c = r.alloc(0, 4 * n + 64) + (shift and 12)
            r.upload(0, b, si.uniform_f32(g, n))
            r.upload(0, c, si.uniform_f32(g, n))
            r.launch(0, gd.GD_K_TRIAD, gd.gd_args_triad(a, b, c, n, -0.625, repeat), mode=mode, **shape)
            r.oracle("triad", 0, a, b, c, -0.625, n, mode=omode)
            assert rel_frobenius(r.download(a, np.float32, n), r.sim.view(a, np.float32, n)) <= FP32_TOL
            r.assert_images_equal(skip=[(a, 4 * n)], what=f"triad repeat={repeat} mode={mode} n={n}")
            once = r.download(a, np.uint32, n).copy()
            r.dview(a, np.uint8, 4 * n).fill_(0)
            r.launch(0, gd.GD_K_TRIAD, gd.gd_args_triad(a, b, c, n, -0.625, 0), mode=mode, **shape)
            assert np.array_equal(r.download(a, np.uint32, n), once)       # bit-identical to the single pass
        torch.cuda.synchronize()
        assert int(counters.sum().item()) == 0
    finally:
        r.close()


@pytest.mark.parametrize("mode", [gd.GD_FENCE_BITWISE, gd.GD_FENCE_MODULO])
def test_copy_triad_with_arrays_split_by_the_partition_end(rig2, mode):
    """16-byte aligned arrays that run over the end of the partition (at a tile boundary, inside a tile,
    inside a vector's neighbourhood) or end exactly there: the fence maps a wrapping array to two ranges,
    so the kernel's test of the whole array fails and every vector is fenced per lane; an array that ends
    at the partition's last byte still takes the per-array fence.  The image equals the oracle's either way."""
    r = rig2
    omode = ok.MODE_BITWISE if mode == gd.GD_FENCE_BITWISE else ok.MODE_MODULO
    base, size = r.row(1)
    g = si.rng(0, 44)
    n = 6000
    for cut in (16, 1024 - 16, 400 * 4, 1024 * 3 + 528, 4 * n):   # bytes of the array in front of the partition end (4n: it ends exactly there)
        lo = r.alloc(1, 64 * KiB)                                  # keeps the partition's first bytes free of inputs
        b, c = r.alloc(1, 4 * n), r.alloc(1, 4 * n)
        r.upload(1, b, si.uniform_f32(g, n))
        r.upload(1, c, si.uniform_f32(g, n))
        a = base + size - cut                                      # output wraps to the partition's first bytes
        r.launch(1, gd.GD_K_TRIAD, gd.gd_args_triad(a, b, c, n, 0.5, 0), mode=mode)
        r.oracle("triad", 1, a, b, c, 0.5, n, mode=omode)
        assert r.sim.last[2] == n - cut // 4
        head, tail = r.download(a, np.float32, cut // 4), r.download(base, np.float32, n - cut // 4)
        want = np.concatenate([r.sim.view(a, np.float32, cut // 4), r.sim.view(base, np.float32, n - cut // 4)])
        assert rel_frobenius(np.concatenate([head, tail]), want) <= FP32_TOL
        r.assert_images_equal(skip=[(a, cut), (base, 4 * n - cut)], what=f"split tile, cut={cut}")
        # a split tile on the input side: copy the wrapped array out again, through aliases one partition off
        r.upload(1, a, r.sim.view(a, np.float32, cut // 4).copy())             # same bits on both sides first
        r.upload(1, base, r.sim.view(base, np.float32, n - cut // 4).copy())
        dst = r.alloc(1, 4 * n)
        r.launch(1, gd.GD_K_COPY, gd.gd_args_copy(dst + size, a - size, n), mode=mode)
        r.oracle("copy", 1, dst + size, a - size, n, mode=omode)
        r.assert_images_equal(what=f"split tile copy, cut={cut}")
        for p in (lo, b, c, dst):
            r.free(1, p)


def test_triad_array_split_on_a_partition_larger_than_4gib():
    """The same on the 64-bit rule (8 GiB partition): values from the oracle on the in-bounds twin of the
    launch, locations from the oracle's fence."""
    r = Rig([8 * GiB], fill=None, simulate=False)
    try:
        base, size = r.row(0)
        g = si.rng(0, 45)
        n = 5000
        cut = 1024 * 2 + 272
        r.alloc(0, 5 * GiB)
        b, c = r.alloc(0, 4 * n), r.alloc(0, 4 * n)
        assert b - base > 4 * GiB
        vb, vc = si.uniform_f32(g, n), si.uniform_f32(g, n)
        r.upload(0, b, vb)
        r.upload(0, c, vc)
        a = base + size - cut
        r.dview(base, np.uint8, 4 * n).fill_(0x5A)
        r.dview(a - 4096, np.uint8, 4096 + cut).fill_(0x5A)
        r.launch(0, gd.GD_K_TRIAD, gd.gd_args_triad(a, b + size, c - size, n, 0.5, 0))
        sim = ok.SimPool(1 << 30, 3 * 4 * n, 0)                   # in-bounds twin: plain addresses, same values
        sa, sb_, sc = sim.pool_base, sim.pool_base + 4 * n, sim.pool_base + 8 * n
        sim.view(sb_, np.float32, n)[:] = vb
        sim.view(sc, np.float32, n)[:] = vc
        sim.run("triad", (sim.pool_base, 1 << 30), ok.MODE_BITWISE, sa, sb_, sc, 0.5, n)
        where = ok.fence_array(base, size, np.uint64(a) + 4 * np.arange(n, dtype=np.uint64), 4)
        assert np.array_equal(where[: cut // 4], a + 4 * np.arange(cut // 4, dtype=np.uint64))
        assert np.array_equal(where[cut // 4:], base + 4 * np.arange(n - cut // 4, dtype=np.uint64))
        got = np.concatenate([r.download(a, np.float32, cut // 4), r.download(base, np.float32, n - cut // 4)])
        assert rel_frobenius(got, sim.view(sa, np.float32, n)) <= FP32_TOL
        assert np.all(r.download(a - 4096, np.uint8, 4096) == 0x5A)                       # nothing in front of the output
        assert np.all(r.download(base + 4 * n - cut, np.uint8, cut) == 0x5A)              # nothing behind its wrapped part
    finally:
        r.close()


def test_indexed_kernels_on_a_partition_larger_than_4gib():
    """Scatter, gather and indexed saxpy on the 64-bit rule (8 GiB partition, arrays above its 4 GiB line), with a
    twentieth of the indices off by whole multiples of the partition size, up and down: the bitwise rule brings each
    of them back to the element the in-range index names, so the result must equal the oracle's on the in-bounds twin
    of the launch (plain addresses, in-range indices, same values), bit for bit for the moved data."""
    r = Rig([8 * GiB], fill=None, simulate=False)
    try:
        base, size = r.row(0)
        g = si.rng(0, 46)
        n = 40003
        per = size // 4
        r.alloc(0, 5 * GiB)
        src, dst, idx, out, x, y, off = (r.alloc(0, 4 * n), r.alloc(0, 4 * n), r.alloc(0, 8 * n), r.alloc(0, 4 * n),
                                         r.alloc(0, 4 * n), r.alloc(0, 4 * n), r.alloc(0, 4 * n))
        assert src - base > 4 * GiB
        vs, vx, vy = si.uniform_f32(g, n), si.uniform_f32(g, n), si.uniform_f32(g, n)
        k0 = g.permutation(n).astype(np.int64)
        far = g.choice(n, size=n // 20, replace=False)
        k = k0.copy()
        k[far] += g.integers(1, 1 << 20, size=far.size) * per * g.choice([-1, 1], size=far.size)
        r.upload(0, src, vs)
        r.upload(0, idx, k)
        r.dview(dst, np.float32, n).zero_()
        # the in-bounds twin
        sim = ok.SimPool(1 << 30, 32 * n, 0)
        t_src, t_dst, t_idx, t_out = (sim.pool_base + 4 * n * j for j in (0, 1, 2, 4))
        sim.view(t_src, np.float32, n)[:] = vs
        sim.view(t_idx, np.int64, n)[:] = k0
        twin = (sim.pool_base, 1 << 30)
        r.launch(0, gd.GD_K_SCATTER_F32_I64, gd.gd_args_scatter(dst, src, idx, n, -1.5, 0))
        sim.run("scatter_f32_i64", twin, ok.MODE_BITWISE, t_dst, t_src, t_idx, -1.5, n)
        assert np.array_equal(r.download(dst, np.float32, n).view(np.uint32), sim.view(t_dst, np.uint32, n))
        r.launch(0, gd.GD_K_GATHER32_I64, gd.gd_args_gather(out, dst, idx, n))
        sim.run("gather32_i64", twin, ok.MODE_BITWISE, t_out, t_dst, t_idx, n)
        assert np.array_equal(r.download(out, np.float32, n).view(np.uint32), sim.view(t_out, np.uint32, n))
        # saxpy: int32 offsets reach +-2^31 elements = 8 GiB = exactly one partition size either way
        o = np.arange(n, dtype=np.int64)
        o[far] += per * g.choice([-1, 1], size=far.size)
        o[o >= 1 << 31] -= 2 * per
        r.upload(0, x, vx)
        r.upload(0, y, vy)
        r.upload(0, off, o.astype(np.int32))
        t_x, t_y, t_off = t_src, t_dst, t_out
        sim.view(t_x, np.float32, n)[:] = vx
        sim.view(t_y, np.float32, n)[:] = vy
        sim.view(t_off, np.int32, n)[:] = np.arange(n, dtype=np.int32)
        r.launch(0, gd.GD_K_SAXPY_IDX, gd.gd_args_saxpy_idx(x, y, off, n, 0.375, 0))
        sim.run("saxpy_idx", twin, ok.MODE_BITWISE, t_x, t_y, t_off, 0.375, n)
        assert rel_frobenius(r.download(y, np.float32, n), sim.view(t_y, np.float32, n)) <= FP32_TOL
        assert np.array_equal(r.download(x, np.float32, n), vx) and np.array_equal(r.download(src, np.float32, n), vs)
    finally:
        r.close()


# ---------------------------------------------------------------------------
# indexed saxpy (configuration 1 shape) with out-of-range offsets
# ---------------------------------------------------------------------------

def hazard_free_offsets(g, n, x, y, scratch, scratch_bytes, base, size, frac=0.01, reach=16 * MiB):
    """Configuration-1 offsets, redrawn (same stream) until every out-of-range
    element's fenced y-address falls into the scratch region, at a location no
    other element uses, and its fenced x-address is not written by this launch.
    Then the final memory image does not depend on the order of the threads."""
    off, where = si.c1_offsets(g, n, y, base, size, frac, reach)
    for _ in range(200):
        o = off[where].astype(np.int64)
        ya = ok.fence_array(base, size, (np.uint64(y) + (4 * o).astype(np.uint64)), 4)
        xa = ok.fence_array(base, size, (np.uint64(x) + (4 * o).astype(np.uint64)), 4)
        in_scratch = (ya >= scratch) & (ya < scratch + scratch_bytes)
        _, first = np.unique(ya, return_index=True)
        dup = np.ones(len(ya), bool)
        dup[first] = False
        x_written = ((xa >= y) & (xa < y + 4 * n)) | np.isin(xa, ya)
        bad = ~in_scratch | dup | x_written
        if not bad.any():
            return off, where
        redo, _ = si.c1_offsets(g, n, y, base, size, frac, reach)
        fresh = redo[redo != np.arange(n)]
        off[where[bad]] = fresh[: bad.sum()]
    raise AssertionError("could not draw hazard-free offsets")


def test_config1_indexed_saxpy_two_tenants_hazard_free_image_is_bit_exact(rig2):
    r = rig2
    n = 262144
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    plan = []
    for t in (0, 1):
        base, size = r.row(t)
        g = si.rng(1, t)
        x, y, off, scratch = (r.alloc(t, 4 * n) for _ in range(4))
        r.upload(t, x, si.uniform_f32(g, n))
        r.upload(t, y, si.uniform_f32(g, n))
        alpha = float(si.uniform_f32(g, 1)[0])
        offs, where = hazard_free_offsets(g, n, x, y, scratch, 4 * n, base, size)
        assert len(where) == 2621
        r.upload(t, off, offs)
        plan.append((t, x, y, off, alpha))
    torch.cuda.synchronize()
    for (t, x, y, off, alpha), st in zip(plan, streams):
        r.launch(t, gd.GD_K_SAXPY_IDX, gd.gd_args_saxpy_idx(x, y, off, n, alpha, 0), stream=st.cuda_stream)
    for (t, x, y, off, alpha) in plan:
        r.oracle("saxpy_idx", t, x, y, off, alpha, n)
        assert r.sim.last[0] == 0 and r.sim.last[2] >= 3 * 2621
    torch.cuda.synchronize()
    got, want = r.image().view(np.float32), r.sim.mem.view(np.float32)
    # every 4-byte word of the pool either matches bit for bit or is a saxpy result
    # that differs in the last place only (fused multiply-add vs fp64 then rounding)
    differ = np.flatnonzero(got.view(np.uint32) != want.view(np.uint32))
    assert np.all(np.isfinite(got[differ])) and np.all(np.isfinite(want[differ]))
    assert np.all(np.abs(got[differ] - want[differ]) <= 2e-7 * np.maximum(1.0, np.abs(want[differ])))
    assert differ.size < 0.01 * n
    for (t, x, y, off, alpha) in plan:
        assert rel_frobenius(r.download(y, np.float32, n), r.sim.view(y, np.float32, n)) <= FP32_TOL


def test_config1_literal_offsets_confinement_and_clean_values():
    # The literal distribution (wrapped stores may hit the tenant's own live data,
    # which the paper leaves unspecified): neighbours stay byte-identical and every
    # element not involved in a wrapped access matches the oracle.
    r = Rig([4 * MiB, 4 * MiB, 4 * MiB])
    try:
        n = 262144
        t = 1
        base, size = r.row(t)
        g = si.rng(1, 7)
        x, y, off = (r.alloc(t, 4 * n) for _ in range(3))
        r.upload(t, x, si.uniform_f32(g, n))
        r.upload(t, y, si.uniform_f32(g, n))
        offs, where = si.c1_offsets(g, n, y, base, size)
        r.upload(t, off, offs)
        before = r.image().copy()
        r.launch(t, gd.GD_K_SAXPY_IDX, gd.gd_args_saxpy_idx(x, y, off, n, 0.5, 0))
        r.oracle("saxpy_idx", t, x, y, off, 0.5, n)
        after = r.image()
        lo, hi = base - r.base, base - r.base + size
        assert np.array_equal(after[:lo], before[:lo]) and np.array_equal(after[hi:], before[hi:])
        o = offs[where].astype(np.int64)
        ya = ok.fence_array(base, size, np.uint64(y) + (4 * o).astype(np.uint64), 4)
        dirty = np.zeros(n, bool)
        dirty[where] = True
        hit_y = ya[(ya >= y) & (ya < y + 4 * n)]
        dirty[((hit_y - y) // 4).astype(np.int64)] = True
        hit_x = ya[(ya >= x) & (ya < x + 4 * n)]
        dirty[((hit_x - x) // 4).astype(np.int64)] = True
        hit_off = ya[(ya >= off) & (ya < off + 4 * n)]
        dirty[((hit_off - off) // 4).astype(np.int64)] = True
        gy, wy = r.download(y, np.float32, n), r.sim.view(y, np.float32, n)
        clean = ~dirty
        assert clean.sum() > 0.95 * n
        # An element whose offset word was overwritten by a wrapped store performs one
        # rogue store at an order-dependent place: at most that many further elements
        # may differ; all others must match.
        close = np.abs(gy - wy) <= 2e-7 * np.maximum(1.0, np.abs(wy))
        assert (clean & ~close).sum() <= len(hit_off)
        assert rel_frobenius(gy[clean & close], wy[clean & close]) <= FP32_TOL
    finally:
        r.close()


# ---------------------------------------------------------------------------
# gather / scatter
# ---------------------------------------------------------------------------

def test_gather_scatter_i64_with_out_of_bounds_indices():
    r = Rig([16 * MiB, 16 * MiB])
    try:
        t = 0
        base, size = r.row(t)
        tab_n, n = 1 << 19, (1 << 19) + 37
        g = si.rng(2, 0)
        tab, idx, out = r.alloc(t, 4 * tab_n), r.alloc(t, 8 * n), r.alloc(t, 4 * n)
        scratch = r.alloc(t, 1 * MiB)
        r.upload(t, tab, si.normal_f32(g, tab_n))
        ix, where = si.c2_indices(g, n, tab_n, frac=0.001, oob_hi=1 << 30)
        # gather has no wrapped stores; only loads that land on `out` (written by this
        # launch) are order-dependent: redraw those
        img = ok.fence_array(base, size, np.uint64(tab) + (4 * ix[where]).astype(np.uint64), 4)
        clash = (img >= out) & (img < out + 4 * n)
        ix[where[clash]] = tab_n + 5
        r.upload(t, idx, ix)
        r.launch(t, gd.GD_K_GATHER32_I64, gd.gd_args_gather(out, tab, idx, n))
        r.oracle("gather32_i64", t, out, tab, idx, n)
        assert r.sim.last[2] >= len(where) - clash.sum()
        r.assert_images_equal(what="gather i64")

        # scatter back, negated.  Out-of-range targets are steered into the scratch
        # region, each to its own word, so the image is order-independent.
        oob_slots = g.choice(MiB // 4, size=len(where), replace=False).astype(np.int64)
        ix[where] = (scratch - tab) // 4 + oob_slots + (size // 4) * g.integers(1, 1 << 20, size=len(where))
        r.upload(t, idx, ix)
        r.launch(t, gd.GD_K_SCATTER_F32_I64, gd.gd_args_scatter(tab, out, idx, n, -1.0, 0))
        # in-bounds duplicates must all carry the same value for the result to be unique:
        # out[i] == tab_old[idx[i]] holds for them by construction of the gather
        r.oracle("scatter_f32_i64", t, tab, out, idx, -1.0, n)
        r.assert_images_equal(what="scatter i64")
        # in-bounds indices only: fenced and unfenced gathers are bit-identical
        ix[where] = 0
        r.upload(t, idx, ix)
        r.launch(t, gd.GD_K_GATHER32_I64, gd.gd_args_gather(out, tab, idx, n))
        a = r.download(out, np.uint32, n).copy()
        r.dview(out, np.uint8, 4 * n).fill_(0)
        r.launch(t, gd.GD_K_GATHER32_I64, gd.gd_args_gather(out, tab, idx, n), mode=gd.GD_FENCE_NONE)
        assert np.array_equal(a, r.download(out, np.uint32, n))
    finally:
        r.close()


@pytest.mark.parametrize("shift", [0, 4])
def test_gather_i32_with_out_of_bounds_and_negative_indices(rig2, shift):
    r = rig2
    t = 1
    base, size = r.row(t)
    tab_n, n = 1 << 18, 200003
    g = si.rng(5, 3)
    tab, idx, out = r.alloc(t, 4 * tab_n), r.alloc(t, 4 * n + 64) + shift, r.alloc(t, 4 * n + 64) + shift
    r.upload(t, tab, g.integers(-2**31, 2**31, size=tab_n, dtype=np.int64).astype(np.int32))
    ix, where = si.c5_indices_i32(g, n, tab_n)
    ix[where[::3]] *= -1
    img = ok.fence_array(base, size, (np.uint64(tab) + (4 * ix[where].astype(np.int64)).astype(np.uint64)), 4)
    clash = (img >= out - 64) & (img < out + 4 * n + 64)
    ix[where[clash]] = tab_n
    r.upload(t, idx, ix)
    r.launch(t, gd.GD_K_GATHER32_I32, gd.gd_args_gather(out, tab, idx, n))
    r.oracle("gather32_i32", t, out, tab, idx, n)
    r.assert_images_equal(what="gather i32")
    fenced = r.download(out, np.int32, n)
    ix[where] = 1
    r.upload(t, idx, ix)
    r.launch(t, gd.GD_K_GATHER32_I32, gd.gd_args_gather(out, tab, idx, n))
    a = r.download(out, np.int32, n)
    r.launch(t, gd.GD_K_GATHER32_I32, gd.gd_args_gather(out, tab, idx, n), mode=gd.GD_FENCE_NONE)
    assert np.array_equal(a, r.download(out, np.int32, n))
    keep = np.ones(n, bool)
    keep[where] = False
    assert np.array_equal(a[keep], fenced[keep])


# ---------------------------------------------------------------------------
# sum, RMSNorm
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("n,shift", [(0, 0), (1, 0), (1000, 0), (4099, 0), (1 << 20, 0), ((1 << 22) + 3, 0), (70001, 4)])
def test_sum_against_fp64(n, shift):
    r = Rig([32 * MiB, 4 * MiB])
    try:
        g = si.rng(5, 1)
        src = r.alloc(0, 4 * n + 64) + shift
        ws, out = r.alloc(0, gd.GD_SUM_WORKSPACE), r.alloc(0, 256)
        r.upload(0, src, si.uniform_f32(g, n, 0.0, 1.0))
        r.launch(0, gd.GD_K_SUM_F32, gd.gd_args_sum(out, src, ws, n))
        exact = r.oracle("sum_f32_exact", 0, src, n)
        r.oracle("sum_f32", 0, out, src, n)
        got = float(r.download(out, np.float32, 1)[0])
        assert abs(got - exact) <= FP32_TOL * max(abs(exact), 1e-30) or (n == 0 and got == 0.0)
        r.assert_images_equal(skip=[(out, 4), (ws, gd.GD_SUM_WORKSPACE)], what="sum")
        r.launch(0, gd.GD_K_SUM_F32, gd.gd_args_sum(out + 16, src, ws, n), mode=gd.GD_FENCE_NONE)
        assert r.download(out + 16, np.float32, 1)[0] == np.float32(got)
        with pytest.raises(gd.GuardianError):
            r.launch(0, gd.GD_K_SUM_F32, gd.gd_args_sum(out, src, ws, n), grid=(4, 1, 1))
    finally:
        r.close()


@pytest.mark.parametrize("rows,cols,shift", [(5, 8192, 0), (33, 4096, 0), (7, 1000, 0), (3, 9000, 0), (4, 8200, 0),
                                             (6, 257, 0), (9, 512, 2), (0, 64, 0), (3, 16384, 0), (5, 12288, 0), (3, 16392, 0), (2, 40008, 0)])
def test_rmsnorm_against_oracle(rows, cols, shift):
    r = Rig([4 * MiB, 4 * MiB])
    try:
        g = si.rng(5, 2)
        x = r.alloc(0, 2 * rows * cols + 64) + shift
        y = r.alloc(0, 2 * rows * cols + 64) + shift
        gain = r.alloc(0, 2 * cols + 64)
        r.upload(0, x, si.f32_to_bf16_bits(si.normal_f32(g, rows * cols)))
        r.upload(0, gain, si.f32_to_bf16_bits(si.uniform_f32(g, cols, 0.5, 1.5)))
        args = gd.gd_args_rmsnorm(y, x, gain, rows, cols, 1e-6, 0)
        r.launch(0, gd.GD_K_RMSNORM_BF16, args)
        r.oracle("rmsnorm_bf16", 0, y, x, gain, rows, cols, 1e-6)
        got = r.download(y, np.uint16, rows * cols)
        want = r.sim.view(y, np.uint16, rows * cols)
        if rows:
            assert rel_frobenius(si.bf16_bits_to_f32(got), si.bf16_bits_to_f32(want)) <= BF16_TOL
            assert np.mean(got != want) < 0.02          # only sparse one-unit flips
        r.assert_images_equal(skip=[(y & ~1, 2 * rows * cols)], what="rmsnorm")
        if shift == 0:
            r.dview(y, np.uint8, 2 * rows * cols).fill_(0)
            r.launch(0, gd.GD_K_RMSNORM_BF16, args, mode=gd.GD_FENCE_NONE)
            assert np.array_equal(r.download(y, np.uint16, rows * cols), got)
    finally:
        r.close()


# ---------------------------------------------------------------------------
# GEMM
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("M,N,K,b_is_nk", [(256, 256, 64, 1), (512, 256, 192, 1), (256, 768, 128, 1), (512, 512, 1024, 1),
                                           (128, 128, 64, 1), (256, 384, 512, 1), (200, 136, 96, 1), (37, 300, 72, 1),
                                           (129, 1, 8, 1), (64, 64, 20, 1), (50, 70, 33, 0), (128, 96, 64, 0),
                                           (16, 16, 0, 1),
                                           # every way the slice ring can end (K/32 mod 10 = 8, 2, 6, 0, 4, 8) and restart
                                           (256, 256, 256, 1), (256, 256, 384, 1), (256, 512, 512, 1), (256, 256, 640, 1),
                                           (512, 256, 768, 1), (256, 256, 896, 1), (256, 256, 1280, 1),
                                           # K % 128 = 64: the ring of K = 64 blocks, every way it can end (K/64 mod 5)
                                           (256, 256, 320, 1), (256, 512, 448, 1), (256, 256, 576, 1),
                                           # a multiple of 8 workgroup tiles (the renumbering over the 8 XCDs is on) and
                                           # more tile rows than one band of GROUP_M = 4, the last band ragged
                                           (2048, 1024, 128, 1), (1280, 2048, 256, 1), (2304, 768, 64, 1)])
def test_gemm_against_oracle(M, N, K, b_is_nk):
    r = Rig([8 * MiB, 4 * MiB])
    try:
        g = si.rng(4, M + N + K)
        A, B, Cc = r.alloc(0, 2 * M * K + 16), r.alloc(0, 2 * K * N + 16), r.alloc(0, 2 * M * N)
        scale = np.float32(1.0 / np.sqrt(max(K, 1)))
        r.upload(0, A, si.f32_to_bf16_bits(si.normal_f32(g, M * K) * scale))
        r.upload(0, B, si.f32_to_bf16_bits(si.normal_f32(g, K * N)))
        args = gd.gd_args_gemm(Cc, A, B, M, N, K, b_is_nk)
        r.launch(0, gd.GD_K_GEMM_BF16, args)
        r.oracle("gemm_bf16", 0, Cc, A, B, M, N, K, b_is_nk, 0, M, 0, N)
        got = r.download(Cc, np.uint16, M * N)
        want = r.sim.view(Cc, np.uint16, M * N)
        assert rel_frobenius(si.bf16_bits_to_f32(got), si.bf16_bits_to_f32(want)) <= BF16_TOL
        assert_bf16_close(got, want, abs_tol=GEMM_ABS_TOL, what=f"gemm {M}x{N}x{K}")
        r.assert_images_equal(skip=[(Cc, 2 * M * N)], what="gemm")
        r.dview(Cc, np.uint8, 2 * M * N).fill_(0)
        r.launch(0, gd.GD_K_GEMM_BF16, args, mode=gd.GD_FENCE_NONE)
        assert np.array_equal(r.download(Cc, np.uint16, M * N), got)
    finally:
        r.close()


def test_gemm_with_wrapping_operand_pointers():
    # A and B addressed through aliases one partition size below: every tile load
    # is redirected to the real operands, C lands where the oracle says.
    r = Rig([8 * MiB, 8 * MiB])
    try:
        t = 1
        base, size = r.row(t)
        M, N, K = 192, 160, 128
        g = si.rng(4, 99)
        A, B, Cc = r.alloc(t, 2 * M * K), r.alloc(t, 2 * K * N), r.alloc(t, 2 * M * N)
        r.upload(t, A, si.f32_to_bf16_bits(si.normal_f32(g, M * K) * np.float32(K ** -0.5)))
        r.upload(t, B, si.f32_to_bf16_bits(si.normal_f32(g, K * N)))
        r.launch(t, gd.GD_K_GEMM_BF16, gd.gd_args_gemm(Cc + size, A - size, B - size, M, N, K, 1))
        r.oracle("gemm_bf16", t, Cc + size, A - size, B - size, M, N, K, 1, 0, M, 0, N)
        got, want = r.download(Cc, np.uint16, M * N), r.sim.view(Cc, np.uint16, M * N)
        assert_bf16_close(got, want, abs_tol=GEMM_ABS_TOL, what="gemm wrapped")
        r.assert_images_equal(skip=[(Cc, 2 * M * N)], what="gemm wrapped")
    finally:
        r.close()


def test_gemm_operands_aligned_to_16_bytes_only():
    """Tile-multiple shape, but A and B are not 128-byte aligned: the launcher must fall back
    from the slice-ring kernel (which relies on that alignment) to the ring of K = 64 blocks."""
    r = Rig([8 * MiB, 4 * MiB])
    try:
        M = N = 256
        K = 256
        g = si.rng(4, 77)
        A, B, Cc = r.alloc(0, 2 * M * K + 256) + 16, r.alloc(0, 2 * K * N + 256) + 48, r.alloc(0, 2 * M * N)
        r.upload(0, A, si.f32_to_bf16_bits(si.normal_f32(g, M * K) * np.float32(K ** -0.5)))
        r.upload(0, B, si.f32_to_bf16_bits(si.normal_f32(g, K * N)))
        args = gd.gd_args_gemm(Cc, A, B, M, N, K, 1)
        r.launch(0, gd.GD_K_GEMM_BF16, args)
        r.oracle("gemm_bf16", 0, Cc, A, B, M, N, K, 1, 0, M, 0, N)
        got = r.download(Cc, np.uint16, M * N)
        want = r.sim.view(Cc, np.uint16, M * N)
        assert_bf16_close(got, want, abs_tol=GEMM_ABS_TOL, what="gemm, 16-byte aligned operands")
        r.assert_images_equal(skip=[(Cc, 2 * M * N)], what="gemm, 16-byte aligned operands")
    finally:
        r.close()


def test_gemm_tile_kernel_with_an_operand_running_past_the_partition_end():
    """Multiples of the tile in every dimension and 128-byte aligned operands: the slice-ring
    kernel, whose DMAs reach the second half of a cache line through the instruction's
    immediate offset.  A starts 64 KiB below the end of the partition, so its rows 128..255
    wrap around to the partition's first bytes; B and C are handed over a whole partition off."""
    r = Rig([8 * MiB, 8 * MiB])
    try:
        t = 1
        base, size = r.row(t)
        M = N = K = 256
        g = si.rng(4, 123)
        low = r.alloc(t, 64 * 1024)                      # first allocation: the partition's first bytes
        assert low == base
        B, Cc = r.alloc(t, 2 * K * N), r.alloc(t, 2 * M * N)
        a_bits = si.f32_to_bf16_bits(si.normal_f32(g, M * K) * np.float32(K ** -0.5))
        A = base + size - 64 * 1024
        r.upload(t, A, a_bits[: M * K // 2])             # rows 0..127 at the top of the partition
        r.upload(t, low, a_bits[M * K // 2:])            # rows 128..255 where the fence sends them
        r.upload(t, B, si.f32_to_bf16_bits(si.normal_f32(g, K * N)))
        args = gd.gd_args_gemm(Cc - size, A, B + size, M, N, K, 1)
        r.launch(t, gd.GD_K_GEMM_BF16, args)
        r.oracle("gemm_bf16", t, Cc - size, A, B + size, M, N, K, 1, 0, M, 0, N)
        got, want = r.download(Cc, np.uint16, M * N), r.sim.view(Cc, np.uint16, M * N)
        assert_bf16_close(got, want, abs_tol=GEMM_ABS_TOL, what="gemm wrapped at the partition end")
        r.assert_images_equal(skip=[(Cc, 2 * M * N)], what="gemm wrapped at the partition end")
        # and it is the product of the matrix as uploaded
        ref = si.bf16_bits_to_f32(a_bits).reshape(M, K).astype(np.float64) @ \
            si.bf16_bits_to_f32(r.download(B, np.uint16, K * N)).reshape(N, K).astype(np.float64).T
        assert rel_frobenius(si.bf16_bits_to_f32(got).reshape(M, N), ref) <= 4e-3
    finally:
        r.close()


# ---------------------------------------------------------------------------
# tenants on concurrent streams; re-carving mid-run
# ---------------------------------------------------------------------------

def test_eight_tenants_on_concurrent_streams_stay_in_their_partitions():
    sizes = [2 * MiB] * 8
    r = Rig(sizes)
    try:
        n = 150001
        streams = [torch.cuda.Stream() for _ in sizes]
        plan = []
        for t in range(8):
            g = si.rng(3, t)
            a, b, c = (r.alloc(t, 4 * n) for _ in range(3))
            r.upload(t, b, si.uniform_f32(g, n))
            r.upload(t, c, si.uniform_f32(g, n))
            plan.append((t, a, b, c, float(si.uniform_f32(g, 1)[0])))
        torch.cuda.synchronize()
        for _ in range(3):
            for (t, a, b, c, s), st in zip(plan, streams):
                # odd tenants misbehave: their pointers are off by whole partitions
                k = (t % 2) * (t + 1) * sizes[t]
                r.launch(t, gd.GD_K_TRIAD, gd.gd_args_triad(a + k, b - k, c + 3 * k, n, s, 0), stream=st.cuda_stream)
                r.launch(t, gd.GD_K_COPY, gd.gd_args_copy(c - k, a + k, n), stream=st.cuda_stream)
        for _ in range(3):
            for (t, a, b, c, s) in plan:
                k = (t % 2) * (t + 1) * sizes[t]
                r.oracle("triad", t, a + k, b - k, c + 3 * k, s, n)
                r.oracle("copy", t, c - k, a + k, n)
        torch.cuda.synchronize()
        got, want = r.image().view(np.float32), r.sim.mem.view(np.float32)
        ok_bits = got.view(np.uint32) == want.view(np.uint32)
        assert rel_frobenius(got[~ok_bits], want[~ok_bits]) <= FP32_TOL if (~ok_bits).any() else True
        assert (~ok_bits).sum() < 0.001 * got.size
    finally:
        r.close()


def test_recarve_mid_run_leaves_other_tenants_untouched():
    sizes = [1 * MiB, 4 * MiB, 2 * MiB, 1 * MiB]
    r = Rig(sizes)
    try:
        n = 60000
        g = si.rng(5, 9)
        bufs = {}
        for t in range(4):
            src, dst = r.alloc(t, 4 * n), r.alloc(t, 4 * n)
            r.upload(t, src, si.uniform_f32(g, n))
            r.launch(t, gd.GD_K_COPY, gd.gd_args_copy(dst, src, n))
            r.oracle("copy", t, dst, src, n)
            bufs[t] = (src, dst)
        r.assert_images_equal(what="before re-carve")
        # tenants 0 and 2 leave a 3 MiB hole: a 4 MiB tenant does not fit...
        for t in (0, 2):
            for p in bufs.pop(t):
                r.free(t, p)
            gd.gd_tenant_detach(r.pool, t)
            assert r.model.detach(t)
        with pytest.raises(gd.GuardianError) as e:
            gd.gd_tenant_attach(r.pool, 4 * MiB)
        assert e.value.status == gd.GD_ENOMEM and r.model.attach(4 * MiB) is None
        # ...but two 512 KiB tenants and a 1 MiB tenant fit
        new = [gd.gd_tenant_attach(r.pool, s) for s in (512 * KiB, 1 * MiB, 512 * KiB)]
        assert new == [r.model.attach(s) for s in (512 * KiB, 1 * MiB, 512 * KiB)]
        for t in new:
            b, s, m = gd.gd_partition_info(r.pool, t)
            assert (b, s) == r.row(t)
            src, dst = r.alloc(t, 4 * 30000), r.alloc(t, 4 * 30000)
            r.upload(t, src, si.uniform_f32(g, 30000))
            # a write-only launch that overruns its (new, smaller) partition on purpose
            r.launch(t, gd.GD_K_STORE_TID, gd.gd_args_store_tid(dst, 200000, 100 + t, 0))
            r.oracle("store_tid", t, dst, 100 + t, 200000)
        r.assert_images_equal(what="after re-carve")
        for t in (1, 3):
            src, dst = bufs[t]
            assert np.array_equal(r.download(dst, np.float32, n), r.sim.view(src, np.float32, n))
    finally:
        r.close()


# ---------------------------------------------------------------------------
# the measurement aids: they compute what they say
# ---------------------------------------------------------------------------

def test_gather_policy_probe_is_a_gather_for_every_policy():
    g = si.rng(0, 60)
    tab_n, n = 1 << 20, (1 << 18) + 4
    tab = torch.from_numpy(g.integers(0, 1 << 32, size=tab_n, dtype=np.uint64).astype(np.uint32).view(np.int32)).cuda()
    idx_h = g.integers(0, tab_n, size=n, dtype=np.int64)
    idx = torch.from_numpy(idx_h).cuda()
    want = tab.cpu().numpy()[idx_h]
    for policy in range(8):
        out = torch.zeros(n, dtype=torch.int32, device="cuda")
        gd.gd_probe_gather_policy(out.data_ptr(), tab.data_ptr(), idx.data_ptr(), n, policy)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), want), policy


def test_mfma_probe_multiplies_what_it_is_given():
    """All operands 1.0 (bf16 0x3F80): every accumulator of the 16x16x32 tiles grows by 32 per instruction and
    the kernel reports acc[0][0][0] + acc[7][7][3]: 2 * 32 * iterations (exact in fp32)."""
    ops = torch.full((16 * 256 * 8,), 0x3F80, dtype=torch.int16, device="cuda")
    blocks, iters = 8, 5
    out = torch.zeros(blocks * 256, dtype=torch.float32, device="cuda")
    gd.gd_probe_mfma(ops.data_ptr(), out.data_ptr(), blocks, iters)
    torch.cuda.synchronize()
    assert torch.all(out == 2.0 * 32.0 * iters).item()
    ops.zero_()
    gd.gd_probe_mfma(ops.data_ptr(), out.data_ptr(), blocks, iters)
    torch.cuda.synchronize()
    assert torch.all(out == 0).item()


def test_host_path_probe_times_three_loops_and_leaves_the_kernels_result(rig2):
    """gd_probe_host_path runs Listing 1's kernel on 64 elements (value 1) through the fenced path and through the
    bare launch call: the image must be what the oracle's single launch leaves, the three per-call times positive,
    and the path that stops before the launch cheaper than the one that launches."""
    r = rig2
    dst = r.alloc(1, 4096)
    for mode, omode in ((gd.GD_FENCE_BITWISE, ok.MODE_BITWISE), (gd.GD_FENCE_NONE, ok.MODE_NONE)):
        up_to, with_launch, bare = gd.gd_probe_host_path(r.pool, 1, dst, 200, mode=mode)
        torch.cuda.synchronize()
        r.oracle("store_tid", 1, dst, 1, 64, mode=omode)
        r.assert_images_equal(what="host path probe")
        assert 0 < up_to < with_launch and 0 < bare, (up_to, with_launch, bare)
        assert up_to < 1e5 and with_launch < 1e6 and bare < 1e6        # nanoseconds per call: sanity only


def test_a_tenant_aiming_every_access_at_its_neighbour_changes_nothing_there(rig2):
    """The threat the paper is about (Sections 1 and 3): tenant 0 passes pointers and indices that all name tenant 1's
    memory -- a store loop over the neighbour's whole partition, a scatter whose every index points into the
    neighbour's live arrays, a gather that tries to read them -- while tenant 1 computes on another stream.  Tenant 1's
    partition must end up exactly as the oracle computes it from tenant 1's own launches; tenant 0 finds its accesses
    redirected into its own partition (and reads back only its own bytes)."""
    r = rig2
    (b0, s0), (b1, s1) = r.row(0), r.row(1)
    g = si.rng(0, 70)
    n = 200000
    va, vb, vc = (r.alloc(1, 4 * n) for _ in range(3))                  # the victim's arrays
    r.upload(1, vb, si.uniform_f32(g, n))
    r.upload(1, vc, si.uniform_f32(g, n))
    src, idx, out = r.alloc(0, 4 * n), r.alloc(0, 8 * n), r.alloc(0, 4 * n)
    secret = r.sim.view(vb, np.float32, n).copy()
    r.upload(0, src, np.full(n, 1234.5, np.float32))
    # indices that, added to tenant 0's own table pointer, name the victim's arrays element by element
    aim = ((vb - src) // 4 + np.arange(n, dtype=np.int64))
    r.upload(0, idx, aim)
    s_att, s_vic = torch.cuda.Stream(), torch.cuda.Stream()
    for rep in range(3):
        r.launch(1, gd.GD_K_TRIAD, gd.gd_args_triad(va, vb, vc, n, 0.5, 0), stream=s_vic.cuda_stream)
        r.launch(0, gd.GD_K_SCATTER_F32_I64, gd.gd_args_scatter(src, src, idx, n, 1.0, 0), stream=s_att.cuda_stream)
        r.launch(0, gd.GD_K_GATHER32_I64, gd.gd_args_gather(out, src, idx, n), stream=s_att.cuda_stream)
        if rep == 0:
            torch.cuda.synchronize()
            stolen = r.download(out, np.float32, n).copy()       # what the aimed gather brought back
        # last, a store loop over the neighbour's whole partition (it wipes the attacker's own arrays instead:
        # the later repetitions attack with whatever indices that leaves)
        r.launch(0, gd.GD_K_STORE_TID, gd.gd_args_store_tid(b1, s1 // 4, 0xDEAD, 0), stream=s_att.cuda_stream)
    torch.cuda.synchronize()
    r.oracle("triad", 1, va, vb, vc, 0.5, n)
    got, want = r.image(), r.sim.mem
    lo, hi, a_lo = b1 - r.base, b1 - r.base + s1, va - r.base
    assert np.array_equal(got[lo:a_lo], want[lo:a_lo]) and np.array_equal(got[a_lo + 4 * n:hi], want[a_lo + 4 * n:hi])
    assert rel_frobenius(r.download(va, np.float32, n), r.sim.view(va, np.float32, n)) <= FP32_TOL
    # the aimed gather read the attacker's own partition: none of the victim's values came back
    assert not np.isin(stolen, secret).any()
    # and the store loop, as long as a partition, ended up covering the attacker's own partition, word for word
    assert (r.download(b0, np.uint32, s0 // 4) == 0xDEAD).all()
