"""ctypes access to ``oracle/gd_oracle.c`` (kernel semantics over a simulated pool).

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).  ``build()`` compiles the
C file with gcc; ``SimPool`` owns the byte array that stands for device memory
and runs the oracle's kernels on it for one tenant at a time.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gd_oracle.c")
_LIB = os.path.join(_HERE, "libgd_oracle.so")
_LIB_OMP = os.path.join(_HERE, "libgd_oracle_omp.so")     # the same file with -fopenmp: timing only

MODE_NONE, MODE_BITWISE, MODE_MODULO, MODE_CHECK, MODE_HWCHECK = 0, 1, 2, 3, 4


# GDO_UBSAN=1 in the environment: every check runs on a build of the same file with gcc's
# undefined-behaviour sanitizer, which aborts the process on the first finding (shifts, signed
# overflow, misaligned or out-of-bounds accesses of the checker itself).
_UBSAN = os.environ.get("GDO_UBSAN") == "1"
_LIB_UBSAN = os.path.join(_HERE, "libgd_oracle_ubsan.so")


def build(force=False, openmp=False):
    """Compile the oracle (plain gcc, -O2, no fast-math).  openmp=False: the sequential
    build every check uses.  openmp=True: its timing twin (see the header of the C file)."""
    out = _LIB_OMP if openmp else (_LIB_UBSAN if _UBSAN else _LIB)
    extra = ["-fopenmp"] if openmp else (
        ["-g", "-fsanitize=undefined", "-fno-sanitize-recover=undefined", "-static-libubsan"] if _UBSAN else [])
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fno-fast-math", "-ffp-contract=off"] + extra + ["-o", out, _SRC, "-lm"])
    return out


class _Ctx(C.Structure):
    _fields_ = [("mem", C.c_void_p), ("pool_base", C.c_uint64), ("pool_bytes", C.c_uint64),
                ("part_base", C.c_uint64), ("part_size", C.c_uint64),
                ("mode", C.c_int32), ("pad", C.c_int32),
                ("escaped", C.c_uint64), ("violations", C.c_uint64), ("wrapped", C.c_uint64)]


_libs = {}


def lib(openmp=False):
    if openmp not in _libs:
        L = C.CDLL(build(openmp=openmp))
        u64, u32, i32, dbl, ctx = C.c_uint64, C.c_uint32, C.c_int32, C.c_double, C.POINTER(_Ctx)
        sigs = {
            "gdo_threads": (C.c_int, []),
            "gdo_fence": (u64, [u64, u64, u64, u32, i32]),
            "gdo_fence_array": (None, [u64, u64, C.c_void_p, u64, u32, i32, C.c_void_p]),
            "gdo_double_to_bf16": (C.c_uint16, [dbl]),
            "gdo_bf16_to_double": (dbl, [C.c_uint16]),
            "gdo_store_tid": (None, [ctx, u64, u32, u64]),
            "gdo_fence_addrs": (None, [ctx, u64, u64, u32, u64]),
            "gdo_chase": (None, [ctx, u64, u64, u64, u64, u32, u32, u32]),
            "gdo_copy": (None, [ctx, u64, u64, u64]),
            "gdo_triad": (None, [ctx, u64, u64, u64, dbl, u64]),
            "gdo_saxpy_idx": (None, [ctx, u64, u64, u64, dbl, u64]),
            "gdo_gather32_i64": (None, [ctx, u64, u64, u64, u64]),
            "gdo_gather32_i32": (None, [ctx, u64, u64, u64, u64]),
            "gdo_scatter_f32_i64": (None, [ctx, u64, u64, u64, dbl, u64]),
            "gdo_sum_f32": (None, [ctx, u64, u64, u64]),
            "gdo_sum_f32_exact": (dbl, [ctx, u64, u64]),
            "gdo_rmsnorm_bf16": (None, [ctx, u64, u64, u64, u64, u64, dbl]),
            "gdo_gemm_bf16": (None, [ctx, u64, u64, u64, u64, u64, u64, i32, u64, u64, u64, u64]),
            "gdo_gemm_bf16_entry": (dbl, [ctx, u64, u64, u64, u64, i32, u64, u64]),
        }
        for name, (res, args) in sigs.items():
            f = getattr(L, name)
            f.restype, f.argtypes = res, args
        _libs[openmp] = L
    return _libs[openmp]


def fence(base, size, addr, width=1, mode=MODE_BITWISE):
    return lib().gdo_fence(base, size, addr, width, mode)


def fence_array(base, size, addrs, width=1, mode=MODE_BITWISE):
    a = np.ascontiguousarray(addrs, dtype=np.uint64)
    out = np.empty_like(a)
    lib().gdo_fence_array(base, size, a.ctypes.data, a.size, width, mode, out.ctypes.data)
    return out


class SimPool:
    """Simulated device memory for ``[pool_base, pool_base + pool_bytes)``.

    ``mem`` is a NumPy uint8 array; ``view(addr, dtype, count)`` gives a typed
    window at a device address (host-side set-up and inspection only -- the
    kernels go through the fence).  ``run(name, tenant_row, mode, *args)`` runs
    one oracle kernel for a tenant whose bounds-table row is ``(base, size)``
    and returns the counters ``(escaped, violations, wrapped)``.
    """

    def __init__(self, pool_base, pool_bytes, fill=0):
        self.pool_base, self.pool_bytes = pool_base, pool_bytes
        self.mem = np.full(pool_bytes, fill, dtype=np.uint8)

    def view(self, addr, dtype, count):
        dtype = np.dtype(dtype)
        off = addr - self.pool_base
        assert 0 <= off and off + count * dtype.itemsize <= self.pool_bytes
        return self.mem[off:off + count * dtype.itemsize].view(dtype)

    def run(self, name, row, mode, *args, openmp=False):
        ctx = _Ctx(self.mem.ctypes.data, self.pool_base, self.pool_bytes, row[0], row[1], mode, 0, 0, 0, 0)
        res = getattr(lib(openmp), "gdo_" + name)(C.byref(ctx), *args)
        self.last = (ctx.escaped, ctx.violations, ctx.wrapped)
        return res if res is not None else self.last
