"""ctypes binding of libguardian.so -- same names as include/guardian.h.

Argument marshalling only.  Functions raise ``GuardianError`` (with ``.status``)
on any status other than GD_OK, except ``gd_check_copy`` which returns the
status, since refusal is its normal answer.  Device addresses are Python ints.
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libguardian.so")

# ---- constants (mirror include/guardian.h) ----------------------------------------
GD_OK, GD_EINVAL, GD_ENOTPOW2, GD_ENOMEM, GD_ERANGE, GD_ENOTENANT, GD_EBUSY, GD_EHIP, \
    GD_ENOKERNEL, GD_ESHAPE = range(10)
GD_FENCE_NONE, GD_FENCE_BITWISE, GD_FENCE_MODULO, GD_FENCE_CHECK, GD_FENCE_HWCHECK = range(5)
(GD_K_STORE_TID, GD_K_FENCE_ADDRS, GD_K_COPY, GD_K_TRIAD, GD_K_SAXPY_IDX, GD_K_GATHER32_I64,
 GD_K_SCATTER_F32_I64, GD_K_GATHER32_I32, GD_K_SUM_F32, GD_K_RMSNORM_BF16, GD_K_GEMM_BF16,
 GD_K_CHASE, GD_K_COUNT) = range(13)
GD_MIN_PARTITION = 4096
GD_GRANULE = 256
GD_SUM_WORKSPACE = 16384
GD_SUM_NOALLOC_MAX_N = 1 << 32

_u64, _u32, _f32 = C.c_uint64, C.c_uint32, C.c_float


def _struct(name, fields):
    return type(name, (C.Structure,), {"_fields_": fields})


gd_args_store_tid = _struct("gd_args_store_tid", [("A", _u64), ("n", _u64), ("j", _u32), ("pad", _u32)])
gd_args_chase = _struct("gd_args_chase", [("out", _u64), ("clk", _u64), ("tab", _u64), ("steps", _u64), ("start", _u32),
                                          ("lane_step", _u32), ("threads", _u32), ("pad", _u32)])
gd_args_fence_addrs = _struct("gd_args_fence_addrs", [("out", _u64), ("in_", _u64), ("n", _u64), ("width", _u32), ("pad", _u32)])
gd_args_copy = _struct("gd_args_copy", [("a", _u64), ("b", _u64), ("n", _u64)])
gd_args_triad = _struct("gd_args_triad", [("a", _u64), ("b", _u64), ("c", _u64), ("n", _u64), ("s", _f32), ("repeat", _u32)])
gd_args_saxpy_idx = _struct("gd_args_saxpy_idx", [("x", _u64), ("y", _u64), ("off", _u64), ("n", _u64), ("alpha", _f32), ("pad", _u32)])
gd_args_gather = _struct("gd_args_gather", [("out", _u64), ("tab", _u64), ("idx", _u64), ("n", _u64)])
gd_args_scatter = _struct("gd_args_scatter", [("dst", _u64), ("src", _u64), ("idx", _u64), ("n", _u64), ("scale", _f32), ("pad", _u32)])
gd_args_sum = _struct("gd_args_sum", [("out", _u64), ("in_", _u64), ("partials", _u64), ("n", _u64)])
gd_args_rmsnorm = _struct("gd_args_rmsnorm", [("y", _u64), ("x", _u64), ("g", _u64), ("rows", _u32), ("cols", _u32), ("eps", _f32), ("pad", _u32)])
gd_args_gemm = _struct("gd_args_gemm", [("C", _u64), ("A", _u64), ("B", _u64), ("M", _u32), ("N", _u32), ("K", _u32), ("b_is_nk", _u32)])

EXPORTS = {
    "gd_pool_create": (C.c_int, [_u64, _u64, C.POINTER(_u64), C.c_int, C.POINTER(C.c_void_p)]),
    "gd_pool_create_flex": (C.c_int, [_u64, _u64, C.POINTER(_u64), C.c_int, C.POINTER(C.c_void_p)]),
    "gd_pool_set_fault_counters": (C.c_int, [C.c_void_p, _u64, C.c_int]),
    "gd_pool_destroy": (C.c_int, [C.c_void_p]),
    "gd_tenant_attach": (C.c_int, [C.c_void_p, _u64, C.POINTER(C.c_int)]),
    "gd_tenant_detach": (C.c_int, [C.c_void_p, C.c_int]),
    "gd_partition_info": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(_u64), C.POINTER(_u64), C.POINTER(_u64)]),
    "gd_alloc": (C.c_int, [C.c_void_p, C.c_int, _u64, _u64, C.POINTER(_u64)]),
    "gd_free": (C.c_int, [C.c_void_p, C.c_int, _u64]),
    "gd_check_copy": (C.c_int, [C.c_void_p, C.c_int, _u64, _u64]),
    "gd_launch_fenced": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_size_t,
                                   C.POINTER(_u32), C.POINTER(_u32), C.c_void_p, C.c_int]),
    "gd_sum_f32_noalloc": (C.c_int, [C.c_void_p, C.c_int, _u64, _u64, _u64, C.c_void_p, C.c_int]),
    "gd_probe_mfma": (C.c_int, [_u64, _u64, _u32, _u32, C.c_void_p]),
    "gd_probe_gather_policy": (C.c_int, [_u64, _u64, _u64, _u64, _u32, C.c_void_p]),
    "gd_probe_host_path": (C.c_int, [C.c_void_p, C.c_int, _u64, _u32, C.c_void_p, C.c_int, C.POINTER(C.c_double)]),
    "gd_kernel_count": (C.c_int, []),
    "gd_kernel_name": (C.c_char_p, [C.c_int]),
    "gd_kernel_args_bytes": (C.c_size_t, [C.c_int]),
    "gd_fence_host": (_u64, [_u64, _u64, _u64, _u32, C.c_int]),
    "gd_strerror": (C.c_char_p, [C.c_int]),
    "gd_last_hip_error": (C.c_int, []),
}

_lib = None


def lib():
    """The loaded library.  No fallback: a missing build is an error."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            f = getattr(L, name)
            f.restype, f.argtypes = res, args
        _lib = L
    return _lib


class GuardianError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        msg = lib().gd_strerror(status).decode()
        if status == GD_EHIP:
            msg += f" (hipError_t {lib().gd_last_hip_error()})"
        super().__init__(f"{what}: {msg}")


def _ok(status, what):
    if status != GD_OK:
        raise GuardianError(status, what)


def gd_pool_create(dev_base, dev_bytes, part_bytes):
    arr = (_u64 * len(part_bytes))(*part_bytes) if len(part_bytes) else None
    out = C.c_void_p()
    _ok(lib().gd_pool_create(dev_base, dev_bytes, arr, len(part_bytes), C.byref(out)), "gd_pool_create")
    return out


def gd_pool_create_flex(dev_base, dev_bytes, part_bytes):
    arr = (_u64 * len(part_bytes))(*part_bytes) if len(part_bytes) else None
    out = C.c_void_p()
    _ok(lib().gd_pool_create_flex(dev_base, dev_bytes, arr, len(part_bytes), C.byref(out)), "gd_pool_create_flex")
    return out


def gd_pool_set_fault_counters(pool, dev_counters, slots):
    _ok(lib().gd_pool_set_fault_counters(pool, dev_counters, slots), "gd_pool_set_fault_counters")


def gd_pool_destroy(pool):
    _ok(lib().gd_pool_destroy(pool), "gd_pool_destroy")


def gd_tenant_attach(pool, nbytes):
    t = C.c_int(-1)
    _ok(lib().gd_tenant_attach(pool, nbytes, C.byref(t)), "gd_tenant_attach")
    return t.value


def gd_tenant_detach(pool, tenant):
    _ok(lib().gd_tenant_detach(pool, tenant), "gd_tenant_detach")


def gd_partition_info(pool, tenant):
    """Returns (base, size, mask)."""
    b, s, m = _u64(), _u64(), _u64()
    _ok(lib().gd_partition_info(pool, tenant, C.byref(b), C.byref(s), C.byref(m)), "gd_partition_info")
    return b.value, s.value, m.value


def gd_alloc(pool, tenant, nbytes, align=GD_GRANULE):
    p = _u64()
    _ok(lib().gd_alloc(pool, tenant, nbytes, align, C.byref(p)), "gd_alloc")
    return p.value


def gd_free(pool, tenant, dptr):
    _ok(lib().gd_free(pool, tenant, dptr), "gd_free")


def gd_check_copy(pool, tenant, dptr, nbytes):
    """Returns the status (GD_OK or GD_ERANGE; GD_ENOTENANT for an unknown tenant)."""
    return lib().gd_check_copy(pool, tenant, dptr, nbytes)


def gd_launch_fenced(pool, tenant, kernel_id, args, stream=None, mode=GD_FENCE_BITWISE, grid=None, block=None):
    """``args`` is one of the gd_args_* structures; ``stream`` a hipStream_t as int (None/0 = null stream)."""
    g = (_u32 * 3)(*grid) if grid is not None else None
    b = (_u32 * 3)(*block) if block is not None else None
    _ok(lib().gd_launch_fenced(pool, tenant, kernel_id, C.byref(args), C.sizeof(args), g, b,
                               C.c_void_p(stream or 0), mode), "gd_launch_fenced")


def gd_sum_f32_noalloc(pool, tenant, out, in_, n, stream=None, mode=GD_FENCE_BITWISE):
    _ok(lib().gd_sum_f32_noalloc(pool, tenant, out, in_, n, C.c_void_p(stream or 0), mode), "gd_sum_f32_noalloc")


def gd_probe_mfma(operands, out, blocks, iters, stream=None):
    _ok(lib().gd_probe_mfma(operands, out, blocks, iters, C.c_void_p(stream or 0)), "gd_probe_mfma")


def gd_probe_gather_policy(out, tab, idx, n, policy, stream=None):
    _ok(lib().gd_probe_gather_policy(out, tab, idx, n, policy, C.c_void_p(stream or 0)), "gd_probe_gather_policy")


def gd_probe_host_path(pool, tenant, dptr, iters, stream=None, mode=GD_FENCE_BITWISE):
    """(ns up to the launch, ns with the launch, ns of the bare HIP launch call), each per call."""
    ns = (C.c_double * 3)()
    _ok(lib().gd_probe_host_path(pool, tenant, dptr, iters, C.c_void_p(stream or 0), mode, ns), "gd_probe_host_path")
    return tuple(ns)


def gd_fence_host(base, size, addr, width=1, mode=GD_FENCE_BITWISE):
    return lib().gd_fence_host(base, size, addr, width, mode)


def gd_kernel_count():
    return lib().gd_kernel_count()


def gd_kernel_name(kernel_id):
    s = lib().gd_kernel_name(kernel_id)
    return s.decode() if s is not None else None


def gd_kernel_args_bytes(kernel_id):
    return lib().gd_kernel_args_bytes(kernel_id)


__all__ = [n for n in dir() if n.startswith(("gd_", "GD_"))] + ["GuardianError", "lib", "LIB_PATH", "EXPORTS"]
