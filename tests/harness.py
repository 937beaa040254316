"""Shared rig for the GPU parity tests: one device pool (a torch uint8 tensor,
aligned by hand), the library's pool over it, and the oracle's simulated pool at
the SAME device addresses, so that pointer and fence arithmetic are identical on
both sides and whole memory images can be compared byte for byte.
"""
import numpy as np
import torch

import paper_2401_09290_amd as gd
from oracle import host_model as hm
from oracle import kernels as ok

KiB, MiB, GiB = 1 << 10, 1 << 20, 1 << 30

NP2TORCH = {np.dtype(np.uint8): torch.uint8, np.dtype(np.int32): torch.int32, np.dtype(np.int64): torch.int64,
            np.dtype(np.float32): torch.float32, np.dtype(np.uint16): torch.int16, np.dtype(np.uint32): torch.int32,
            np.dtype(np.uint64): torch.int64, np.dtype(np.int16): torch.int16}


class Rig:
    """sizes: partition sizes per tenant.  window: bytes of each partition that the
    oracle simulates (None = all of it); accesses of the oracle outside the window
    are counted as escaped, so a test that uses a window asserts there are none."""

    def __init__(self, sizes, fill=0xA5, simulate=True):
        self.sizes = list(sizes)
        biggest = max(sizes)
        total = sum(sizes)
        self.buf = torch.empty(total + biggest, dtype=torch.uint8, device="cuda")
        raw = self.buf.data_ptr()
        self.base = -(-raw // biggest) * biggest
        self.bytes = total
        self.dev = self.buf[self.base - raw:self.base - raw + total]
        self.pool = gd.gd_pool_create(self.base, total, self.sizes)
        self.model = hm.Pool(self.base, total, self.sizes)
        for t in range(len(sizes)):
            b, s, m = gd.gd_partition_info(self.pool, t)
            assert (b, s) == self.model.table[t] and m == hm.partition_mask(b, s)
        self.fill = fill
        if fill is not None:
            self.dev.fill_(fill)
        self.sim = ok.SimPool(self.base, total, fill or 0) if simulate else None
        torch.cuda.synchronize()

    def close(self):
        gd.gd_pool_destroy(self.pool)
        self.pool = None
        self.buf = self.dev = self.sim = None
        torch.cuda.empty_cache()

    def row(self, tenant):
        return self.model.table[tenant]

    def alloc(self, tenant, nbytes, align=256):
        p = gd.gd_alloc(self.pool, tenant, nbytes, align)
        assert p == self.model.heaps[tenant].alloc(nbytes, align)
        return p

    def free(self, tenant, ptr):
        gd.gd_free(self.pool, tenant, ptr)
        assert self.model.heaps[tenant].free(ptr)

    def dview(self, ptr, dtype, count):
        dtype = np.dtype(dtype)
        off = ptr - self.base
        return self.dev[off:off + count * dtype.itemsize].view(NP2TORCH[dtype])

    def upload(self, tenant, ptr, array):
        """Checked host-to-device copy (Section 4.2.2) mirrored into the simulated pool."""
        array = np.ascontiguousarray(array)
        assert gd.gd_check_copy(self.pool, tenant, ptr, array.nbytes) == gd.GD_OK
        src = torch.from_numpy(array.view(np.uint8).reshape(-1))
        self.dview(ptr, np.uint8, array.nbytes).copy_(src)
        if self.sim is not None:
            self.sim.view(ptr, array.dtype, array.size)[:] = array.reshape(-1)

    def download(self, ptr, dtype, count):
        return self.dview(ptr, dtype, count).cpu().numpy().view(dtype)

    def launch(self, tenant, kid, args, mode=gd.GD_FENCE_BITWISE, stream=None, **kw):
        gd.gd_launch_fenced(self.pool, tenant, kid, args, stream=stream, mode=mode, **kw)

    def oracle(self, name, tenant, *args, mode=ok.MODE_BITWISE):
        return self.sim.run(name, self.row(tenant), mode, *args)

    def image(self):
        torch.cuda.synchronize()
        return self.dev.cpu().numpy()

    def assert_images_equal(self, skip=(), what=""):
        """Device pool == simulated pool byte for byte, except the (ptr, nbytes) ranges in skip."""
        got, want = self.image(), self.sim.mem
        if skip:
            got, want = got.copy(), want.copy()
            for (p, n) in skip:
                got[p - self.base:p - self.base + n] = 0
                want[p - self.base:p - self.base + n] = 0
        if not np.array_equal(got, want):
            bad = np.flatnonzero(got != want)
            raise AssertionError(f"{what}: {bad.size} bytes differ, first at pool offset {hex(int(bad[0]))} "
                                 f"(device {got[bad[0]]:#x}, oracle {want[bad[0]]:#x})")


def rel_frobenius(got, ref):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    den = np.linalg.norm(ref)
    return np.linalg.norm(got - ref) / (den if den else 1.0)


def bf16_bits_to_f64(h):
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def assert_bf16_close(got_bits, want_bits, abs_tol=0.0, flip_budget=0.02, frobenius=True, what=""):
    """bf16 output against the oracle's bf16 output, element by element.

    The kernel accumulates in fp32 and the oracle in fp64, so a result that falls next
    to a rounding boundary may land on the neighbouring bf16 value: every element must
    be within ONE bf16 unit in the last place of the oracle's value (2^-7 relative)
    plus `abs_tol` (the fp32 accumulation error, which matters for entries near zero),
    at most `flip_budget` of the elements may differ at all, and the relative
    Frobenius error stays within 1e-3 (`frobenius=False` when the caller passes only
    the elements that differ, whose norm says nothing)."""
    got, want = bf16_bits_to_f64(got_bits).reshape(-1), bf16_bits_to_f64(want_bits).reshape(-1)
    assert got.shape == want.shape
    if got.size == 0:
        return
    err = np.abs(got - want)
    bound = 2.0 ** -7 * np.abs(want) + abs_tol
    worst = int(np.argmax(err - bound))
    assert err[worst] <= bound[worst], f"{what}: element {worst}: got {got[worst]!r}, oracle {want[worst]!r}"
    flips = float(np.mean(np.asarray(got_bits).reshape(-1) != np.asarray(want_bits).reshape(-1)))
    assert flips <= flip_budget, f"{what}: {flips:.4f} of the elements differ from the oracle"
    if frobenius:
        assert rel_frobenius(got, want) <= 1e-3, what
