"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py
times (same kernels, same library-chosen launch shapes, tenants on their own
streams).  Where the pool is too large to simulate whole, the oracle works on a
window that covers everything the tenant's launch can touch (all accesses are
in bounds there; the oracle's `escaped` counter proves it), or on sampled
outputs it computes one by one.
"""
import numpy as np
import pytest
import torch

import paper_2401_09290_amd as gd
import synth_inputs as si
from harness import assert_bf16_close, GiB, MiB, Rig, rel_frobenius
from oracle import kernels as ok

pytestmark = pytest.mark.gpu

FP32_TOL = 1e-5
BF16_TOL = 1e-3


def test_config3_copy_triad_eight_tenants_16gib_partitions():
    n = 1 << 28
    r = Rig([16 * GiB] * 8, fill=None, simulate=False)
    try:
        streams = [torch.cuda.Stream() for _ in range(8)]
        host = {}
        plan = []
        for t in range(8):
            a, b, c = (r.alloc(t, 4 * n) for _ in range(3))
            keep = t in (0, 5)                                  # these two are checked in full
            hb, hc = np.empty(n, np.float32), np.empty(n, np.float32)
            si.fill_chunked(hb, 3, t + 100, "uniform", threads=16)
            si.fill_chunked(hc, 3, t + 200, "uniform", threads=16)
            r.upload(t, b, hb)
            r.upload(t, c, hc)
            s = float(si.uniform_f32(si.rng(3, t), 1)[0])
            rs = np.random.Generator(np.random.PCG64(t))
            pick = np.sort(rs.choice(n, size=200000, replace=False))
            pick[:8] = np.arange(8)
            pick[-8:] = n - 8 + np.arange(8)
            host[t] = (hb, hc) if keep else (hb[pick].copy(), hc[pick].copy())
            plan.append((t, a, b, c, s, keep, pick))
        torch.cuda.synchronize()
        a2 = {t: r.alloc(t, 4 * n) for t in range(8)}
        for (t, a, b, c, s, keep, pick), st in zip(plan, streams):
            r.launch(t, gd.GD_K_COPY, gd.gd_args_copy(a2[t], b, n), stream=st.cuda_stream)
            r.launch(t, gd.GD_K_TRIAD, gd.gd_args_triad(a, b, c, n, s, 0), stream=st.cuda_stream)
        torch.cuda.synchronize()
        for (t, a, b, c, s, keep, pick) in plan:
            base, size = r.row(t)
            assert size == 16 * GiB and base % size == 0
            hb, hc = host[t]
            m = hb.size
            # oracle window: three arrays of m elements at the head of a 16 GiB partition
            sim = ok.SimPool(base, 3 * 4 * m, 0)
            sa, sb, sc = base, base + 4 * m, base + 8 * m
            sim.view(sb, np.float32, m)[:] = hb
            sim.view(sc, np.float32, m)[:] = hc
            assert sim.run("triad", (base, size), ok.MODE_BITWISE, sa, sb, sc, s, m) == (0, 0, 0)
            want = sim.view(sa, np.float32, m)
            got_tri = r.download(a, np.float32, n)
            got_cpy = r.download(a2[t], np.float32, n)
            if not keep:
                got_tri, got_cpy = got_tri[pick], got_cpy[pick]
            assert rel_frobenius(got_tri, want) <= FP32_TOL, f"tenant {t}"
            assert np.max(np.abs(got_tri - want)) <= 2.4e-7
            sim.run("copy", (base, size), ok.MODE_BITWISE, sa, sb, m)
            assert np.array_equal(got_cpy.view(np.uint32), sim.view(sa, np.uint32, m)), f"tenant {t}"
            del sim, got_tri, got_cpy
        # fenced and unfenced builds agree bit for bit (tenant 3, full arrays)
        t, a, b, c, s, _, _ = plan[3]
        fenced = r.dview(a, np.float32, n).clone()
        r.dview(a, np.float32, n).zero_()
        r.launch(t, gd.GD_K_TRIAD, gd.gd_args_triad(a, b, c, n, s, 0), mode=gd.GD_FENCE_NONE)
        torch.cuda.synchronize()
        assert torch.equal(fenced.view(torch.int32), r.dview(a, np.float32, n).view(torch.int32))
    finally:
        r.close()


def test_config2_gather_scatter_one_gib_partition_with_canary_neighbour():
    n = tab_n = 1 << 26
    r = Rig([GiB, GiB], fill=None)
    try:
        t = 0
        base, size = r.row(t)
        nb_base, nb_size = r.row(1)
        canary = si.address_canary(nb_size // 8)
        r.upload(1, nb_base, canary)
        tab, idx, out = r.alloc(t, 4 * tab_n), r.alloc(t, 8 * n), r.alloc(t, 4 * n)
        assert (tab, idx, out) == (base, base + 256 * MiB, base + 768 * MiB)     # partition exactly full
        vals = np.empty(tab_n, np.float32)
        si.fill_chunked(vals, 2, 1, "normal", threads=16)
        r.upload(t, tab, vals)
        ix, where = si.c2_indices(si.rng(2, 0), n, tab_n)
        assert len(where) == 67109 and ix[where].min() >= tab_n and ix[where].max() < (1 << 30)
        r.upload(t, idx, ix)
        r.dview(out, np.uint8, 4 * n).zero_()
        r.sim.view(out, np.uint8, 4 * n)[:] = 0
        torch.cuda.synchronize()

        # ---- gather: loads only wrap; a wrapped load that lands on `out` reads data
        # written by the same launch and is excluded, everything else is bit-exact
        r.launch(t, gd.GD_K_GATHER32_I64, gd.gd_args_gather(out, tab, idx, n))
        r.oracle("gather32_i64", t, out, tab, idx, n)
        # indices below 2^28 still address the tenant's own partition (the index array or `out`)
        assert r.sim.last[0] == 0 and r.sim.last[2] == int((4 * ix[where] >= size).sum())
        img = ok.fence_array(base, size, np.uint64(tab) + (4 * ix[where]).astype(np.uint64), 4)
        assert img.min() >= base and img.max() < base + size
        racy = where[(img >= out) & (img < out + 4 * n)]
        got = r.download(out, np.uint32, n)
        want = r.sim.view(out, np.uint32, n)
        same = got == want
        assert same[np.setdiff1d(np.arange(n), racy, assume_unique=True)].all()
        assert 0.2 * len(where) < len(racy) < 0.3 * len(where)          # `out` is a quarter of the partition
        assert np.array_equal(r.download(nb_base, np.uint64, nb_size // 8), canary)
        # make both sides agree on `out` before the scatter reads it
        r.upload(t, out, want.copy())

        # ---- scatter back, negated, literal index distribution
        r.launch(t, gd.GD_K_SCATTER_F32_I64, gd.gd_args_scatter(tab, out, idx, n, -1.0, 0))
        r.oracle("scatter_f32_i64", t, tab, out, idx, -1.0, n)
        torch.cuda.synchronize()
        assert np.array_equal(r.download(nb_base, np.uint64, nb_size // 8), canary)   # neighbour untouched
        # first-order bookkeeping: words a wrapped store lands on, elements whose index
        # or source word is such a word (their own store then goes to an order-dependent place)
        w_words = (img - np.uint64(base)) // np.uint64(4)
        hit = np.zeros(size // 4, bool)
        hit[w_words.astype(np.int64)] = True
        idx_w0 = (idx - base) // 4
        src_w0 = (out - base) // 4
        dirty_elem = hit[idx_w0:idx_w0 + 2 * n:2] | hit[idx_w0 + 1:idx_w0 + 2 * n:2] | hit[src_w0:src_w0 + n]
        dirty_elem[where] = True
        # table words that only clean in-bounds elements write (or nobody writes)
        unsure = hit[:tab_n].copy()
        unsure[ix[dirty_elem & (ix < tab_n)]] = True
        got_tab = r.download(tab, np.uint32, tab_n)
        want_tab = r.sim.view(tab, np.uint32, tab_n)
        bad = (got_tab != want_tab) & ~unsure
        # a dirty element's rogue store may land on any word: at most one further word each
        # (one on the GPU, one in the oracle's sequential order)
        assert bad.sum() <= 2 * (dirty_elem.sum() - len(where)), (int(bad.sum()), int(dirty_elem.sum()))
        assert (~unsure).mean() > 0.99
        # and the bulk is the negated gather
        clean = ~unsure
        k = np.flatnonzero(clean)[:: 97]
        touched = np.zeros(tab_n, bool)
        touched[ix[ix < tab_n]] = True
        expect = np.where(touched[k], -vals[k], vals[k])
        # (a rogue store that both orders perform identically shows up here and not in `bad`)
        off = got_tab[k].view(np.float32) != expect
        assert off.sum() <= 2 * (dirty_elem.sum() - len(where)) and off.mean() < 1e-3
    finally:
        r.close()


def test_config4_gemm_8192_sampled_entries_and_slab():
    M = N = K = 8192
    r = Rig([4 * GiB], fill=None, simulate=False)
    try:
        A, B, Cc = (r.alloc(0, 2 * M * K) for _ in range(3))
        base, size = r.row(0)
        host = np.empty(M * K, np.float32)
        si.fill_chunked(host, 4, 1, "normal", threads=16)
        Ab = si.f32_to_bf16_bits(host * np.float32(K ** -0.5))
        si.fill_chunked(host, 4, 2, "normal", threads=16)
        Bb = si.f32_to_bf16_bits(host)
        del host
        r.upload(0, A, Ab)
        r.upload(0, B, Bb)
        st = torch.cuda.Stream()
        r.launch(0, gd.GD_K_GEMM_BF16, gd.gd_args_gemm(Cc, A, B, M, N, K, 1), stream=st.cuda_stream)
        torch.cuda.synchronize()
        got = r.download(Cc, np.uint16, M * N).reshape(M, N)
        # oracle window: A and B at their real addresses (C is never stored: entries are returned)
        sim = ok.SimPool(base, 2 * 2 * M * K, 0)
        sim.view(A, np.uint16, M * K)[:] = Ab
        sim.view(B, np.uint16, K * N)[:] = Bb
        # Stratified sample: 8 entries in each of the 32 x 32 workgroup tiles (256 x 256), chosen so that
        # every accumulator slot of the kernel -- wavefront (2 x 2), MFMA tile (8 x 8), lane group (4),
        # register (4): 4096 classes -- is hit twice over the matrix; the lane's row inside its 16 is random.
        g = np.random.Generator(np.random.PCG64(44))
        ms, ns = [], []
        for tile in range(1024):
            tm, tn = divmod(tile, 32)
            for k in range(8):
                slot = (8 * tile + k) % 4096
                wave, i, j, lg, reg = slot >> 10, (slot >> 7) & 7, (slot >> 4) & 7, (slot >> 2) & 3, slot & 3
                ms.append(256 * tm + 128 * (wave >> 1) + 16 * i + int(g.integers(0, 16)))
                ns.append(256 * tn + 128 * (wave & 1) + 16 * j + 4 * lg + reg)
        ms = np.concatenate([ms, [0, 0, M - 1, M - 1, 127, 128, 255, 256]])
        ns = np.concatenate([ns, [0, N - 1, 0, N - 1, 128, 127, 256, 255]])
        exact = np.array([sim.run("gemm_bf16_entry", (base, size), ok.MODE_BITWISE, A, B, N, K, 1, int(m), int(n))
                          for m, n in zip(ms, ns)])
        assert sim.last[0] == 0
        want_bits = np.array([ok.lib().gdo_double_to_bf16(float(e)) for e in exact], dtype=np.uint16)
        assert_bf16_close(got[ms, ns], want_bits, abs_tol=3e-5, what="gemm 8192^3, stratified sample")
        have = si.bf16_bits_to_f32(got[ms, ns]).astype(np.float64)
        assert np.all(np.abs(have - exact) <= 2.0**-8 * np.abs(exact) * 1.01 + 1e-4)   # within one rounding of exact
        # The whole matrix against the second reference: NumPy's fp64 matmul of the same bf16 values,
        # rounded to bf16 (float64 -> float32 -> bf16; the double rounding can move a tie by one unit,
        # which the one-unit bound covers).  Every one of the 67 M entries is checked.
        ref = si.bf16_bits_to_f32(Ab).reshape(M, K).astype(np.float64) @ si.bf16_bits_to_f32(Bb).reshape(N, K).astype(np.float64).T
        ref_bits = si.f32_to_bf16_bits(ref.astype(np.float32).reshape(-1))
        assert np.mean(ref_bits.reshape(M, N)[ms, ns] != want_bits) < 0.01      # the two references agree on the sample
        del ref
        for r0 in range(0, M, 1024):                                              # in slabs: keeps the temporaries small
            assert_bf16_close(got[r0:r0 + 1024], ref_bits.reshape(M, N)[r0:r0 + 1024], abs_tol=3e-5,
                              what=f"gemm 8192^3 vs NumPy, rows {r0}..")
        del ref_bits
        # a slab of whole rows, computed entry by entry by the oracle's kernel
        rows = (0, 4097)
        for m0 in rows:
            sim2 = ok.SimPool(base, 3 * 2 * M * K, 0)
            sim2.view(A, np.uint16, M * K)[:] = Ab
            sim2.view(B, np.uint16, K * N)[:] = Bb
            sim2.run("gemm_bf16", (base, size), ok.MODE_BITWISE, Cc, A, B, M, N, K, 1, m0, m0 + 2, 0, N)
            want_rows = sim2.view(Cc + 2 * m0 * N, np.uint16, 2 * N)
            assert rel_frobenius(si.bf16_bits_to_f32(got[m0:m0 + 2].reshape(-1)), si.bf16_bits_to_f32(want_rows)) <= BF16_TOL
            del sim2
        # protection off gives the same bits
        r.dview(Cc, np.uint8, 2 * M * N).zero_()
        r.launch(0, gd.GD_K_GEMM_BF16, gd.gd_args_gemm(Cc, A, B, M, N, K, 1), mode=gd.GD_FENCE_NONE)
        torch.cuda.synchronize()
        assert np.array_equal(r.download(Cc, np.uint16, M * N).reshape(M, N), got)
    finally:
        r.close()


def test_config5_mixed_tenants_full_size_kernels_and_recarve():
    g = si.rng(5, 0)
    sizes = si.c5_partition_sizes(g, 16, budget=128 * GiB)
    assert max(sizes) >= GiB and all(s & (s - 1) == 0 and 256 * MiB <= s <= 8 * GiB for s in sizes)
    r = Rig(sizes, fill=None, simulate=False)
    try:
        streams = [torch.cuda.Stream() for _ in sizes]
        n_sum, rows, cols, n_g = 1 << 27, 4096, 8192, 1 << 24
        big = [t for t, s in enumerate(sizes) if s >= GiB]
        small = [t for t, s in enumerate(sizes) if s < GiB] or big
        t_sum, t_rms, t_gat = big[0], small[0], small[-1] if small[-1] != small[0] else big[-1]
        checks = []

        # sum
        src, ws, out = r.alloc(t_sum, 4 * n_sum), r.alloc(t_sum, gd.GD_SUM_WORKSPACE), r.alloc(t_sum, 256)
        v = np.empty(n_sum, np.float32)
        si.fill_chunked(v, 5, t_sum + 1, "uniform", 0.0, 1.0, threads=16)
        r.upload(t_sum, src, v)
        r.launch(t_sum, gd.GD_K_SUM_F32, gd.gd_args_sum(out, src, ws, n_sum), stream=streams[t_sum].cuda_stream)
        # RMSNorm
        gt = si.rng(5, t_rms + 1)
        x, y, gain = r.alloc(t_rms, 2 * rows * cols), r.alloc(t_rms, 2 * rows * cols), r.alloc(t_rms, 2 * cols)
        xb = si.f32_to_bf16_bits(si.normal_f32(gt, rows * cols))
        gb = si.f32_to_bf16_bits(si.uniform_f32(gt, cols, 0.5, 1.5))
        r.upload(t_rms, x, xb)
        r.upload(t_rms, gain, gb)
        r.launch(t_rms, gd.GD_K_RMSNORM_BF16, gd.gd_args_rmsnorm(y, x, gain, rows, cols, 1e-6, 0), stream=streams[t_rms].cuda_stream)
        # int32 gather, 0.5 % out of bounds
        gt = si.rng(5, t_gat + 1)
        tab, idx, gout = (r.alloc(t_gat, 4 * n_g) for _ in range(3))
        tv = gt.integers(-2**31, 2**31, size=n_g, dtype=np.int64).astype(np.int32)
        ix, where = si.c5_indices_i32(gt, n_g, n_g)
        assert len(where) == 83886
        r.upload(t_gat, tab, tv)
        r.upload(t_gat, idx, ix)
        r.dview(gout, np.uint8, 4 * n_g).zero_()
        r.launch(t_gat, gd.GD_K_GATHER32_I32, gd.gd_args_gather(gout, tab, idx, n_g), stream=streams[t_gat].cuda_stream)
        torch.cuda.synchronize()

        # ---- oracle, tenant by tenant, on windows at the real addresses
        base, size = r.row(t_sum)
        sim = ok.SimPool(base, out + 256 - base, 0)
        sim.view(src, np.float32, n_sum)[:] = v
        exact = sim.run("sum_f32_exact", (base, size), ok.MODE_BITWISE, src, n_sum)
        got = float(r.download(out, np.float32, 1)[0])
        assert abs(got - exact) <= FP32_TOL * exact and abs(exact - n_sum / 2) < 1e-3 * n_sum
        del sim, v

        base, size = r.row(t_rms)
        sim = ok.SimPool(base, gain + 2 * cols - base, 0)
        sim.view(x, np.uint16, rows * cols)[:] = xb
        sim.view(gain, np.uint16, cols)[:] = gb
        sim.run("rmsnorm_bf16", (base, size), ok.MODE_BITWISE, y, x, gain, rows, cols, 1e-6)
        assert sim.last[0] == 0
        gy, wy = r.download(y, np.uint16, rows * cols), sim.view(y, np.uint16, rows * cols)
        assert rel_frobenius(si.bf16_bits_to_f32(gy), si.bf16_bits_to_f32(wy)) <= BF16_TOL
        assert np.mean(gy != wy) < 0.02
        del sim

        base, size = r.row(t_gat)
        assert (tab, idx, gout) == (base, base + 4 * n_g, base + 8 * n_g)
        sim = ok.SimPool(base, 3 * 4 * n_g, 0)
        sim.view(tab, np.int32, n_g)[:] = tv
        sim.view(idx, np.int32, n_g)[:] = ix
        sim.run("gather32_i32", (base, size), ok.MODE_BITWISE, gout, tab, idx, n_g)
        img = ok.fence_array(base, size, np.uint64(tab) + (4 * ix[where].astype(np.int64)).astype(np.uint64), 4)
        # a wrapped load is checkable if it lands on the table or the indices (uploaded data);
        # on `gout` it races with this launch's stores, elsewhere the partition was never written
        checkable = img < gout
        keep = np.ones(n_g, bool)
        keep[where[~checkable]] = False
        assert checkable.sum() > 1000
        gg, wg = r.download(gout, np.int32, n_g), sim.view(gout, np.int32, n_g)
        assert np.array_equal(gg[keep], wg[keep])
        # and every in-bounds element is the table entry
        inb = np.ones(n_g, bool)
        inb[where] = False
        assert np.array_equal(gg[inb], tv[ix[inb]])
        del sim

        # ---- re-carve: the gather tenant leaves and returns smaller/larger; others keep their data
        before_sum = r.download(src, np.float32, 4096).copy()
        for p in (tab, idx, gout):
            r.free(t_gat, p)
        gd.gd_tenant_detach(r.pool, t_gat)
        assert r.model.detach(t_gat)
        new_size = 512 * MiB if sizes[t_gat] != 512 * MiB else 256 * MiB
        try:
            nt = gd.gd_tenant_attach(r.pool, new_size)
        except gd.GuardianError:
            new_size = sizes[t_gat]
            nt = gd.gd_tenant_attach(r.pool, new_size)
        assert nt == r.model.attach(new_size) == t_gat
        nb, ns, nm = gd.gd_partition_info(r.pool, nt)
        assert (nb, ns) == r.row(nt) and nb % ns == 0
        p = r.alloc(nt, 4096)
        # a store loop twice as long as the new partition: wraps, stays inside
        guard_lo = r.download(nb - 4096, np.uint8, 4096).copy() if nb - 4096 >= r.base else None
        r.launch(nt, gd.GD_K_STORE_TID, gd.gd_args_store_tid(p, 2 * ns // 4, 0xC0FFEE, 0))
        torch.cuda.synchronize()
        assert bool((r.dview(nb, np.int32, ns // 4) == 0xC0FFEE).all().item())
        if guard_lo is not None:
            assert np.array_equal(r.download(nb - 4096, np.uint8, 4096), guard_lo)
        assert np.array_equal(r.download(src, np.float32, 4096), before_sum)
        assert float(r.download(out, np.float32, 1)[0]) == got
    finally:
        r.close()


def test_copy_triad_and_sum_of_more_than_2_pow_32_elements():
    """Maximum sizes: arrays of 2^32 + 1027 fp32 elements (16 GiB each) in a 64 GiB partition, so that element
    indices, byte offsets and tile counts all pass 2^32.  The values are an address-dependent pattern made on the
    device; the whole result is compared on the device with what the definition gives (copy: the same bits; triad:
    one fused multiply-add per element, the kernel's own precision), and the oracle recomputes sampled windows --
    the first MiB, and the MiB in front of element 2^32 together with everything behind it -- from the bytes the kernel read."""
    n = (1 << 32) + 1027
    r = Rig([64 * GiB], fill=None, simulate=False)
    try:
        base, size = r.row(0)
        a, b, c = (r.alloc(0, 4 * n) for _ in range(3))
        chunk = 1 << 28
        for p, salt in ((b, 0x9E3779B1), (c, 0x85EBCA77)):
            view = r.dview(p, np.float32, n)
            for lo in range(0, n, chunk):
                hi = min(n, lo + chunk)
                i = torch.arange(lo, hi, dtype=torch.int64, device="cuda")
                view[lo:hi] = (((i * salt) >> 7) & 0xFFFFF).to(torch.float32) * (1.0 / (1 << 19)) - 1.0     # exact in fp32, in [-1, 1)
                del i
        r.dview(a, np.uint8, 4 * n).fill_(0x5A)
        s = 0.6180339887
        windows = [(0, 1 << 18), ((1 << 32) - (1 << 18), (1 << 18) + 1027)]      # the second one crosses element 2^32 and ends with the arrays
        for kid, args, oname in ((gd.GD_K_COPY, gd.gd_args_copy(a, b, n), "copy"), (gd.GD_K_TRIAD, gd.gd_args_triad(a, b, c, n, s, 0), "triad")):
            r.launch(0, kid, args)
            torch.cuda.synchronize()
            va, vb, vc = (r.dview(p, np.float32, n) for p in (a, b, c))
            for lo in range(0, n, chunk):
                hi = min(n, lo + chunk)
                if oname == "copy":
                    assert torch.equal(va[lo:hi].view(torch.int32), vb[lo:hi].view(torch.int32)), (oname, lo)
                else:
                    want = torch.addcmul(vb[lo:hi].double(), vc[lo:hi].double(), torch.tensor(s, dtype=torch.float32, device="cuda").double()).float()
                    assert torch.equal(va[lo:hi], want), (oname, lo)        # fp64 product and sum rounded once = the fused multiply-add
                    del want
            for (lo, cnt) in windows:
                sim = ok.SimPool(1 << 30, 3 * 4 * cnt, 0)
                sa, sb, sc = sim.pool_base, sim.pool_base + 4 * cnt, sim.pool_base + 8 * cnt
                sim.view(sb, np.float32, cnt)[:] = r.download(b + 4 * lo, np.float32, cnt)
                sim.view(sc, np.float32, cnt)[:] = r.download(c + 4 * lo, np.float32, cnt)
                if oname == "copy":
                    sim.run("copy", (sim.pool_base, 1 << 30), ok.MODE_BITWISE, sa, sb, cnt)
                    assert np.array_equal(r.download(a + 4 * lo, np.uint32, cnt), sim.view(sa, np.uint32, cnt)), (oname, lo)
                else:
                    sim.run("triad", (sim.pool_base, 1 << 30), ok.MODE_BITWISE, sa, sb, sc, float(np.float32(s)), cnt)
                    assert rel_frobenius(r.download(a + 4 * lo, np.float32, cnt), sim.view(sa, np.float32, cnt)) <= FP32_TOL, (oname, lo)
            r.dview(a, np.uint8, 4 * n).fill_(0x5A)
        # the sum over the same 2^32 + 1027 values (grid-stride loop past 2^32): against the fp64 sum taken chunk by chunk
        # on the device; the values are centred on zero, so the bound is relative to the sum of magnitudes
        ws, out = r.alloc(0, gd.GD_SUM_WORKSPACE), r.alloc(0, 256)
        r.launch(0, gd.GD_K_SUM_F32, gd.gd_args_sum(out, b, ws, n))
        torch.cuda.synchronize()
        vb = r.dview(b, np.float32, n)
        exact = sum(float(vb[lo:min(n, lo + chunk)].double().sum().item()) for lo in range(0, n, chunk))
        magnitude = sum(float(vb[lo:min(n, lo + chunk)].double().abs().sum().item()) for lo in range(0, n, chunk))
        got = float(r.download(out, np.float32, 1)[0])
        assert abs(got - exact) <= FP32_TOL * magnitude, (got, exact, magnitude)
        assert abs(exact) > 1.0                                  # a zero result would pass the bound for the wrong reason
    finally:
        r.close()
