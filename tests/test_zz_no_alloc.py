"""The allocation-free sum (gd_sum_f32_noalloc) against the existing entry point
(gd_launch_fenced with GD_K_SUM_F32 and a tenant workspace): same bits, on two calls
in a row, the second with a smaller input; every fence variant; the size limit."""
import numpy as np
import pytest
import torch

import paper_2401_09290_amd as gd
import synth_inputs as si
from harness import GiB, MiB, Rig

pytestmark = pytest.mark.gpu


def test_noalloc_sum_matches_the_workspace_sum_bit_for_bit():
    r = Rig([64 * MiB, 4 * MiB], simulate=False)
    try:
        counters = torch.zeros(4, dtype=torch.int64, device="cuda")
        gd.gd_pool_set_fault_counters(r.pool, counters.data_ptr(), 4)
        g = si.rng(5, 70)
        n_big, n_small = (1 << 23) + 12345, 70001           # 2049 and 18 workgroups: the second call reads fewer partials
        src = r.alloc(0, 4 * n_big)
        ws, ref, out = r.alloc(0, gd.GD_SUM_WORKSPACE), r.alloc(0, 256), r.alloc(0, 256)
        r.upload(0, src, si.uniform_f32(g, n_big, 0.0, 1.0))
        st = torch.cuda.Stream()
        for mode in (gd.GD_FENCE_BITWISE, gd.GD_FENCE_NONE, gd.GD_FENCE_MODULO, gd.GD_FENCE_CHECK):
            for n, in_ptr in ((n_big, src), (n_small, src + 4 * 1000), (0, src), (5, src + 4)):
                r.dview(ref, np.uint32, 1).fill_(0x7FC00001)
                r.dview(out, np.uint32, 1).fill_(0x7FC00002)
                r.launch(0, gd.GD_K_SUM_F32, gd.gd_args_sum(ref, in_ptr, ws, n), mode=mode, stream=st.cuda_stream)
                gd.gd_sum_f32_noalloc(r.pool, 0, out, in_ptr, n, stream=st.cuda_stream, mode=mode)
                torch.cuda.synchronize()
                a, b = int(r.download(ref, np.uint32, 1)[0]), int(r.download(out, np.uint32, 1)[0])
                assert a == b, (mode, n, hex(a), hex(b))
                if n:
                    want = float(r.download(in_ptr, np.float32, n).astype(np.float64).sum())
                    assert abs(float(np.uint32(b).view(np.float32)) - want) <= 1e-5 * want
        # wrapped pointers go through the tenant's fence exactly as in the existing entry point
        base, size = r.row(0)
        r.launch(0, gd.GD_K_SUM_F32, gd.gd_args_sum(ref + size, src - size, ws, n_small), stream=st.cuda_stream)
        gd.gd_sum_f32_noalloc(r.pool, 0, out - size, src + size, n_small, stream=st.cuda_stream)
        torch.cuda.synchronize()
        assert int(r.download(ref, np.uint32, 1)[0]) == int(r.download(out, np.uint32, 1)[0])
        assert int(counters.sum().item()) == 0
        # sizes beyond the stated maximum are refused before anything is launched
        with pytest.raises(gd.GuardianError) as e:
            gd.gd_sum_f32_noalloc(r.pool, 0, out, src, gd.GD_SUM_NOALLOC_MAX_N + 1)
        assert e.value.status == gd.GD_ESHAPE
        with pytest.raises(gd.GuardianError) as e:
            gd.gd_sum_f32_noalloc(r.pool, 7, out, src, 16)
        assert e.value.status == gd.GD_ENOTENANT
    finally:
        r.close()
