"""Host half of the C ABI, checked against the oracle without a GPU: the library
loads, exports what include/guardian.h declares, and its partition table,
allocator, range check and host fence agree with oracle/host_model.py
address for address.  No kernel is launched here.
"""
import ctypes as C
import os
import random
import re

import pytest

import paper_2401_09290_amd as gd
from oracle import host_model as hm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
KiB, MiB, GiB = 1 << 10, 1 << 20, 1 << 30


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "guardian.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(gd_[a-z_0-9]+)\s*\(", header))
    assert {"gd_pool_create", "gd_alloc", "gd_free", "gd_check_copy", "gd_launch_fenced"} <= declared
    raw = C.CDLL(gd.LIB_PATH)
    for name in declared:
        assert hasattr(raw, name), name
    assert declared == set(gd.EXPORTS)


def test_registry_matches_argument_blocks():
    blocks = {
        gd.GD_K_STORE_TID: gd.gd_args_store_tid, gd.GD_K_FENCE_ADDRS: gd.gd_args_fence_addrs,
        gd.GD_K_COPY: gd.gd_args_copy, gd.GD_K_TRIAD: gd.gd_args_triad,
        gd.GD_K_SAXPY_IDX: gd.gd_args_saxpy_idx, gd.GD_K_GATHER32_I64: gd.gd_args_gather,
        gd.GD_K_SCATTER_F32_I64: gd.gd_args_scatter, gd.GD_K_GATHER32_I32: gd.gd_args_gather,
        gd.GD_K_SUM_F32: gd.gd_args_sum, gd.GD_K_RMSNORM_BF16: gd.gd_args_rmsnorm,
        gd.GD_K_GEMM_BF16: gd.gd_args_gemm, gd.GD_K_CHASE: gd.gd_args_chase,
    }
    assert gd.gd_kernel_count() == gd.GD_K_COUNT == len(blocks)
    names = set()
    for kid, struct in blocks.items():
        assert gd.gd_kernel_args_bytes(kid) == C.sizeof(struct), gd.gd_kernel_name(kid)
        names.add(gd.gd_kernel_name(kid))
    assert len(names) == len(blocks)
    assert gd.gd_kernel_name(-1) is None and gd.gd_kernel_name(gd.GD_K_COUNT) is None
    assert gd.gd_kernel_args_bytes(99) == 0


def test_partition_info_reproduces_printed_example(golden):
    (base, size, end, mask), = golden("section4_3_mask_example.txt")
    base, size, end, mask = int(base, 16), int(size), int(end, 16), int(mask, 16)
    pool = gd.gd_pool_create(base, size, [size])
    b, s, m = gd.gd_partition_info(pool, 0)
    assert (b, s, m) == (base, size, mask) and b + s - 1 == end
    gd.gd_pool_destroy(pool)


def test_pool_create_places_partitions_like_the_oracle():
    rnd = random.Random(21)
    for _ in range(300):
        sizes = [1 << rnd.randint(12, 34) for _ in range(rnd.randint(0, 16))]
        pool_base = rnd.randrange(1, 1 << 20) * 4096
        slack = rnd.choice([0, 0, max(sizes, default=0)])
        pool_bytes = sum(sizes) + slack
        want = hm.carve(pool_base, pool_bytes, sizes)
        if want is None:
            with pytest.raises(gd.GuardianError) as e:
                gd.gd_pool_create(pool_base, pool_bytes, sizes)
            assert e.value.status == gd.GD_ENOMEM
            continue
        pool = gd.gd_pool_create(pool_base, pool_bytes, sizes)
        for t, (b, s) in enumerate(want):
            assert gd.gd_partition_info(pool, t) == (b, s, s - 1)
        gd.gd_pool_destroy(pool)


def test_pool_create_rejects_bad_requests():
    for sizes, status in (([3 * MiB], gd.GD_ENOTPOW2), ([2048], gd.GD_ENOTPOW2), ([0], gd.GD_ENOTPOW2),
                          ([MiB, MiB + 1], gd.GD_ENOTPOW2), ([2 * MiB], gd.GD_ENOMEM)):
        with pytest.raises(gd.GuardianError) as e:
            gd.gd_pool_create(16 * MiB, MiB, sizes)
        assert e.value.status == status
    with pytest.raises(gd.GuardianError) as e:
        gd.gd_pool_create((1 << 64) - 4096, 8192, [4096])          # range wraps the address space
    assert e.value.status == gd.GD_EINVAL
    pool = gd.gd_pool_create(16 * MiB, MiB, [])
    with pytest.raises(gd.GuardianError) as e:
        gd.gd_partition_info(pool, 0)
    assert e.value.status == gd.GD_ENOTENANT
    gd.gd_pool_destroy(pool)


def test_attach_detach_follow_the_oracle_and_never_move_others():
    rnd = random.Random(5)
    base, nbytes = 1 << 30, 1 << 26
    sizes = [1 << 22, 1 << 24, 1 << 20]
    pool, model = gd.gd_pool_create(base, nbytes, sizes), hm.Pool(base, nbytes, sizes)
    for _ in range(400):
        live = [t for t, r in enumerate(model.table) if r]
        if live and rnd.random() < 0.5:
            t = rnd.choice(live)
            assert model.detach(t)
            gd.gd_tenant_detach(pool, t)
            with pytest.raises(gd.GuardianError) as e:
                gd.gd_partition_info(pool, t)
            assert e.value.status == gd.GD_ENOTENANT
        else:
            size = 1 << rnd.randint(12, 25)
            want = model.attach(size)
            if want is None:
                with pytest.raises(gd.GuardianError) as e:
                    gd.gd_tenant_attach(pool, size)
                assert e.value.status == gd.GD_ENOMEM
            else:
                assert gd.gd_tenant_attach(pool, size) == want
        for t, row in enumerate(model.table):
            if row:
                assert gd.gd_partition_info(pool, t) == (row[0], row[1], row[1] - 1)
    gd.gd_pool_destroy(pool)


def test_detach_is_refused_while_allocations_live():
    pool = gd.gd_pool_create(1 << 30, 1 << 22, [1 << 20, 1 << 20])
    p = gd.gd_alloc(pool, 1, 100)
    with pytest.raises(gd.GuardianError) as e:
        gd.gd_tenant_detach(pool, 1)
    assert e.value.status == gd.GD_EBUSY
    gd.gd_free(pool, 1, p)
    gd.gd_tenant_detach(pool, 1)
    with pytest.raises(gd.GuardianError) as e:
        gd.gd_alloc(pool, 1, 100)
    assert e.value.status == gd.GD_ENOTENANT
    gd.gd_pool_destroy(pool)


def test_alloc_free_traces_match_the_oracle_address_for_address():
    rnd = random.Random(13)
    base = 0x7FA2D0000000
    sizes = [256 * KiB, 64 * KiB]
    pool, model = gd.gd_pool_create(base, sum(sizes), sizes), hm.Pool(base, sum(sizes), sizes)
    live = {0: [], 1: []}
    for _ in range(6000):
        t = rnd.randint(0, 1)
        if live[t] and rnd.random() < 0.45:
            p = live[t].pop(rnd.randrange(len(live[t])))
            assert model.heaps[t].free(p)
            gd.gd_free(pool, t, p)
            with pytest.raises(gd.GuardianError) as e:            # double free
                gd.gd_free(pool, t, p)
            assert e.value.status == gd.GD_EINVAL
            continue
        nbytes, align = rnd.randint(1, 20000), 1 << rnd.randint(0, 13)
        want = model.heaps[t].alloc(nbytes, align)
        if want is None:
            with pytest.raises(gd.GuardianError) as e:
                gd.gd_alloc(pool, t, nbytes, align)
            assert e.value.status == gd.GD_ENOMEM
        else:
            got = gd.gd_alloc(pool, t, nbytes, align)
            assert got == want
            b, s, _ = gd.gd_partition_info(pool, t)
            assert b <= got and got + nbytes <= b + s and got % max(align, 256) == 0
            live[t].append(got)
    for t in live:
        for p in live[t]:
            gd.gd_free(pool, t, p)
        b, s, _ = gd.gd_partition_info(pool, t)
        assert gd.gd_alloc(pool, t, s) == b                        # fully coalesced again
    with pytest.raises(gd.GuardianError) as e:
        gd.gd_free(pool, 0, gd.gd_partition_info(pool, 1)[0])      # another tenant's pointer
    assert e.value.status == gd.GD_EINVAL
    for bad in ((0, 256), (16, 3), (16, 0)):
        with pytest.raises(gd.GuardianError) as e:
            gd.gd_alloc(pool, 0, *bad)
        assert e.value.status == gd.GD_EINVAL
    gd.gd_pool_destroy(pool)


def test_check_copy_grid_matches_set_inclusion():
    base = 1 << 20
    sizes = [8 * KiB, 4 * KiB, 4 * KiB]
    pool = gd.gd_pool_create(base, 16 * KiB, sizes)
    table = hm.carve(base, 16 * KiB, sizes)
    for t, (b, s) in enumerate(table):
        for p in range(base - 4 * KiB, base + 20 * KiB, 128):
            for n in (0, 1, 127, 128, 4 * KiB - 128, 4 * KiB, 4 * KiB + 1, 8 * KiB, 8 * KiB + 128, 16 * KiB):
                want = gd.GD_OK if hm.check_copy(b, s, p, n) else gd.GD_ERANGE
                assert gd.gd_check_copy(pool, t, p, n) == want, (t, hex(p), n)
    b, s = table[0]
    assert gd.gd_check_copy(pool, 0, (1 << 64) - 8, 64) == gd.GD_ERANGE
    assert gd.gd_check_copy(pool, 0, b + 8, (1 << 64) - 1) == gd.GD_ERANGE
    assert gd.gd_check_copy(pool, 0, b + s, 0) == gd.GD_OK
    assert gd.gd_check_copy(pool, 7, b, 1) == gd.GD_ENOTENANT
    # bounds of the partition, not of the allocation: a range over free space is accepted
    gd.gd_alloc(pool, 0, 256)
    assert gd.gd_check_copy(pool, 0, b + 4096, 1024) == gd.GD_OK
    gd.gd_pool_destroy(pool)


@pytest.mark.parametrize("width", hm.ACCESS_WIDTHS)
def test_host_fence_equals_oracle_on_tiny_pool_and_random_addresses(width):
    sizes = [4 * KiB, 32 * KiB, 8 * KiB, 4 * KiB, 16 * KiB]
    pool_base, pool_bytes = 0x40000, 64 * KiB
    rnd = random.Random(width)
    for (b, s) in hm.carve(pool_base, pool_bytes, sizes):
        for a in range(pool_base - pool_bytes, pool_base + 2 * pool_bytes, 3):
            assert gd.gd_fence_host(b, s, a, width) == hm.fence(a, b, s, width)
    for _ in range(20000):
        s = 1 << rnd.randint(12, 40)
        b = s * rnd.randint(1, 1 << 12)
        a = rnd.getrandbits(64)
        assert gd.gd_fence_host(b, s, a, width, gd.GD_FENCE_BITWISE) == hm.fence(a, b, s, width)
        assert gd.gd_fence_host(b, s, a, width, gd.GD_FENCE_MODULO) == hm.fence_modulo(a, b, s, width)
        ok = hm.check_access(a, b, s, width)
        assert gd.gd_fence_host(b, s, a, width, gd.GD_FENCE_CHECK) == (a if ok else hm.U64)
        assert gd.gd_fence_host(b, s, a, width, gd.GD_FENCE_NONE) == a
        if s < (1 << 32):
            assert gd.gd_fence_host(b, s, a, width, gd.GD_FENCE_HWCHECK) == (hm.fence_hwcheck(a, b, s, width) or hm.U64)
            near = b + rnd.randint(-2 * s, 3 * s)
            assert gd.gd_fence_host(b, s, near, width, gd.GD_FENCE_HWCHECK) == (hm.fence_hwcheck(near, b, s, width) or hm.U64)
        else:
            assert gd.gd_fence_host(b, s, a, width, gd.GD_FENCE_HWCHECK) == hm.U64     # the rule needs a size below 4 GiB
    assert gd.gd_fence_host(4096 + 256, 4096, 0, 4) == hm.U64           # base not size-aligned
    assert gd.gd_fence_host(4096, 4096, 0, 3) == hm.U64                 # not an access width


def test_flex_pool_places_odd_sizes_like_the_oracle():
    rnd = random.Random(31)
    for _ in range(200):
        sizes = [256 * rnd.randint(16, 5000) for _ in range(rnd.randint(1, 9))]
        pool_base = 256 * rnd.randint(1, 1 << 20) + rnd.choice([0, 0, 8, 100])
        pool_bytes = sum(sizes) + rnd.choice([0, 256, 4096])
        want = hm.carve_flex(pool_base, pool_bytes, sizes)
        if want is None:
            with pytest.raises(gd.GuardianError) as e:
                gd.gd_pool_create_flex(pool_base, pool_bytes, sizes)
            assert e.value.status == gd.GD_ENOMEM
            continue
        pool = gd.gd_pool_create_flex(pool_base, pool_bytes, sizes)
        for t, (b, s) in enumerate(want):
            assert gd.gd_partition_info(pool, t)[:2] == (b, s)
            assert b % 256 == 0 and pool_base <= b and b + s <= pool_base + pool_bytes
        spans = sorted(want)
        for (b0, s0), (b1, _) in zip(spans, spans[1:]):
            assert b0 + s0 <= b1
        # the bitwise fence is refused on such a pool (its partitions are not size-aligned powers of two)
        with pytest.raises(gd.GuardianError) as e:
            gd.gd_launch_fenced(pool, 0, gd.GD_K_COPY, gd.gd_args_copy(want[0][0], want[0][0] + 1024, 4))
        assert e.value.status == gd.GD_EINVAL
        gd.gd_pool_destroy(pool)
    for bad in ([4096 + 8], [2048], [0]):
        with pytest.raises(gd.GuardianError) as e:
            gd.gd_pool_create_flex(1 << 20, 1 << 20, bad)
        assert e.value.status == gd.GD_ENOTPOW2


def test_modulo_host_fence_on_odd_partitions_confines_whole_access():
    rnd = random.Random(17)
    for _ in range(20000):
        size = 256 * rnd.randint(16, 1 << 24)
        base = 256 * rnd.randint(1, 1 << 30)
        a = rnd.getrandbits(64)
        w = rnd.choice(hm.ACCESS_WIDTHS)
        f = gd.gd_fence_host(base, size, a, w, gd.GD_FENCE_MODULO)
        assert f == hm.fence_modulo(a, base, size, w)
        assert base <= f and f + w <= base + size
        if base <= a and a + w <= base + size and a % w == 0:
            assert f == a


def test_fault_counters_must_lie_outside_the_pool():
    pool = gd.gd_pool_create(1 << 30, 1 << 20, [1 << 20])
    for addr in ((1 << 30), (1 << 30) + (1 << 20) - 8, (1 << 30) - 8):
        with pytest.raises(gd.GuardianError) as e:
            gd.gd_pool_set_fault_counters(pool, addr, 4)
        assert e.value.status == gd.GD_EINVAL
    with pytest.raises(gd.GuardianError):
        gd.gd_pool_set_fault_counters(pool, (1 << 29) + 4, 1)            # not 8-byte aligned
    # checking needs the counters
    with pytest.raises(gd.GuardianError) as e:
        gd.gd_launch_fenced(pool, 0, gd.GD_K_COPY, gd.gd_args_copy(1 << 30, (1 << 30) + 4096, 4), mode=gd.GD_FENCE_CHECK)
    assert e.value.status == gd.GD_EINVAL
    gd.gd_pool_set_fault_counters(pool, (1 << 30) + (1 << 20), 1)        # right behind the pool is fine
    gd.gd_pool_set_fault_counters(pool, 1 << 29, 4)
    gd.gd_pool_destroy(pool)


def test_launch_argument_errors_need_no_gpu():
    pool = gd.gd_pool_create(1 << 30, 1 << 20, [1 << 20])
    args = gd.gd_args_copy(1 << 30, (1 << 30) + 4096, 16)
    for tenant, kid, a, status in ((3, gd.GD_K_COPY, args, gd.GD_ENOTENANT),
                                   (0, 99, args, gd.GD_ENOKERNEL),
                                   (0, gd.GD_K_TRIAD, args, gd.GD_EINVAL)):
        with pytest.raises(gd.GuardianError) as e:
            gd.gd_launch_fenced(pool, tenant, kid, a)
        assert e.value.status == status
    with pytest.raises(gd.GuardianError) as e:
        gd.gd_launch_fenced(pool, 0, gd.GD_K_COPY, args, mode=17)
    assert e.value.status == gd.GD_ENOKERNEL
    gd.gd_pool_destroy(pool)
    # the hardware-checked rule addresses a partition through a 32-bit byte count: 4 GiB and more are refused
    pool = gd.gd_pool_create(1 << 40, 1 << 33, [1 << 32, 1 << 31])
    with pytest.raises(gd.GuardianError) as e:
        gd.gd_launch_fenced(pool, 0, gd.GD_K_COPY, gd.gd_args_copy(1 << 40, (1 << 40) + 4096, 16), mode=gd.GD_FENCE_HWCHECK)
    assert e.value.status == gd.GD_ESHAPE
    gd.gd_pool_destroy(pool)


def test_measurement_aids_refuse_bad_arguments_without_a_gpu():
    """The measurement aids validate their arguments before any launch."""
    for args in ((0, 4096, 1, 1), (4096, 0, 1, 1), (4096 + 8, 8192, 1, 1), (4096, 8192 + 2, 1, 1), (4096, 8192, 0, 1),
                 (4096, 8192, 1 << 20, 1)):
        with pytest.raises(gd.GuardianError) as e:
            gd.gd_probe_mfma(*args)
        assert e.value.status == gd.GD_EINVAL
    for args in ((0, 4096, 8192, 16, 0), (4096, 0, 8192, 16, 0), (4096, 8192, 0, 16, 0), (4096 + 4, 8192, 16384, 16, 0),
                 (4096, 8192 + 2, 16384, 16, 0), (4096, 8192, 16384 + 8, 16, 0), (4096, 8192, 16384, 18, 0),
                 (4096, 8192, 16384, 16, 8)):
        with pytest.raises(gd.GuardianError) as e:
            gd.gd_probe_gather_policy(*args)
        assert e.value.status == gd.GD_EINVAL
    gd.gd_probe_gather_policy(4096, 8192, 16384, 0, 3)          # nothing to do: no launch, no GPU needed
    # gd_probe_host_path: arguments and the tenant's row are checked before the first HIP call
    pool = gd.gd_pool_create(1 << 40, 1 << 24, [1 << 22, 1 << 22])
    for args, status in (((0, 0, 1 << 40, 10), gd.GD_EINVAL), ((pool, 0, 0, 10), gd.GD_EINVAL), ((pool, 0, 1 << 40, 0), gd.GD_EINVAL),
                         ((pool, 0, 1 << 40, (1 << 20) + 1), gd.GD_EINVAL), ((pool, 7, 1 << 40, 10), gd.GD_ENOTENANT)):
        with pytest.raises(gd.GuardianError) as e:
            gd.gd_probe_host_path(*args)
        assert e.value.status == status, args
    with pytest.raises(gd.GuardianError) as e:
        gd.gd_probe_host_path(pool, 0, 1 << 40, 10, mode=gd.GD_FENCE_CHECK)      # no fault counters registered
    assert e.value.status == gd.GD_EINVAL
    gd.gd_pool_destroy(pool)


def test_pool_is_safe_to_use_from_several_threads(tmp_path):
    """The header promises one lock per pool: tests/native/pool_threads.cpp drives alloc / free / range checks /
    bounds-table reads / attach / detach from eight threads, built together with csrc/pool.cpp under the thread
    sanitizer and under the address + undefined-behaviour sanitizers (host code only); it checks disjointness, confinement and full coalescing itself."""
    import shutil
    import subprocess
    if shutil.which("g++") is None:
        pytest.skip("needs g++")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    for flags, options in ((["-fsanitize=thread"], {"TSAN_OPTIONS": "halt_on_error=1 exitcode=66"}),
                           (["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"], {"ASAN_OPTIONS": "exitcode=67"})):
        exe = str(tmp_path / ("pool_threads" + flags[0].split("=")[1].split(",")[0]))
        build = subprocess.run(["g++", "-O1", "-g", *flags, "-std=c++17", "-o", exe,
                                os.path.join(root, "tests", "native", "pool_threads.cpp"),
                                os.path.join(root, "paper_2401_09290_amd", "csrc", "pool.cpp"), "-lpthread"],
                               capture_output=True, text=True)
        if build.returncode != 0 and re.search(r"cannot find -l(tsan|asan|ubsan)", build.stderr):
            pytest.skip("sanitizer runtime not installed")
        assert build.returncode == 0, build.stderr
        run = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=dict(os.environ, **options))
        assert run.returncode == 0, (flags, run.returncode, run.stdout[-2000:], run.stderr[-4000:])
        assert "failures 0" in run.stdout


def test_host_allocation_failures_come_back_as_status_codes_and_lose_nothing(tmp_path):
    """tests/native/abi_nothrow.cpp replaces operator new with one that fails on the k-th allocation and calls the
    entry points that allocate (gd_pool_create, gd_alloc, gd_free, gd_tenant_attach) through the built library with
    k = 0, 1, 2, ...: every failing call must return GD_ENOMEM with its out-parameter untouched, nothing may abort,
    and afterwards the whole partition must still be allocatable as one block."""
    import shutil
    import subprocess
    if shutil.which("g++") is None:
        pytest.skip("needs g++")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    libdir = os.path.join(root, "paper_2401_09290_amd")
    gd.lib()                                                   # fails loudly if the library is not built
    exe = str(tmp_path / "abi_nothrow")
    build = subprocess.run(["g++", "-O1", "-g", "-std=c++17", "-o", exe, os.path.join(root, "tests", "native", "abi_nothrow.cpp"),
                            "-L" + libdir, "-lguardian", "-Wl,-rpath," + libdir], capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    run = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0, (run.returncode, run.stdout[-2000:], run.stderr[-4000:])
    assert "problems 0" in run.stdout and "injected" in run.stdout
    injected = int(run.stdout.split("injected")[1].split()[0])
    assert injected >= 8                                       # failures really were injected at several points
