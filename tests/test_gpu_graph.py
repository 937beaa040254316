"""gd_launch_fenced under HIP graph capture: the entry point allocates nothing and
synchronises nothing, so a caller may record fenced launches into a graph (the way to
run launch-bound loops of small kernels).  Every replay is checked against the oracle,
with the program's own eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

import paper_2401_09290_amd as gd
import synth_inputs as si
from harness import MiB, Rig, rel_frobenius

pytestmark = pytest.mark.gpu
FP32_TOL = 1e-5


def test_fenced_launches_recorded_in_a_graph_replay_to_the_oracle_image():
    r = Rig([4 * MiB, 4 * MiB, 4 * MiB])
    try:
        n = 200003
        plan = []
        for t in (0, 1):
            g = si.rng(3, 50 + t)
            a, b, c = (r.alloc(t, 4 * n) for _ in range(3))
            r.upload(t, b, si.uniform_f32(g, n))
            r.upload(t, c, si.uniform_f32(g, n))
            plan.append((t, a, b, c, float(si.uniform_f32(g, 1)[0])))
        size1 = r.row(1)[1]
        d = r.alloc(1, 4 * n)                       # written by a kernel that runs past its end

        def launches(stream):
            for (t, a, b, c, s) in plan:
                # tenant 1 hands over pointers that are whole partitions off: the fence brings them home
                k = size1 if t == 1 else 0
                r.launch(t, gd.GD_K_TRIAD, gd.gd_args_triad(a + k, b - k, c + 2 * k, n, s, 0), stream=stream)
            r.launch(1, gd.GD_K_STORE_TID, gd.gd_args_store_tid(d, n + 5000, 7, 0), stream=stream)

        for (t, a, b, c, s) in plan:
            k = size1 if t == 1 else 0
            r.oracle("triad", t, a + k, b - k, c + 2 * k, float(s), n)
        r.oracle("store_tid", 1, d, 7, n + 5000)

        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            launches(torch.cuda.current_stream().cuda_stream)
        want = r.sim.mem
        for replay in range(3):
            # eager work of the program between the replays: wipe what the graph writes
            for (t, a, b, c, s) in plan:
                r.dview(a, np.uint8, 4 * n).fill_(0)
            r.dview(d, np.uint8, 4 * (n + 5000)).fill_(0xEE)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            got = r.image()
            for (t, a, b, c, s) in plan:
                assert rel_frobenius(r.download(a, np.float32, n), r.sim.view(a, np.float32, n)) <= FP32_TOL, (replay, t)
            skip = [(a, 4 * n) for (t, a, b, c, s) in plan]
            g2, w2 = got.copy(), want.copy()
            for (p, nb) in skip:
                g2[p - r.base:p - r.base + nb] = 0
                w2[p - r.base:p - r.base + nb] = 0
            assert np.array_equal(g2, w2), f"replay {replay}: bytes outside the triad results differ"
    finally:
        r.close()


def test_every_kind_of_kernel_and_the_allocation_free_sum_replay_from_a_graph():
    """One graph holding a gather, a scatter, the two-pass sum, the allocation-free sum (the entry point meant for
    callers under capture), an RMSNorm and an MFMA GEMM: every replay, with eager wipes of all outputs in between,
    must reproduce what the oracle computes for the same launches."""
    from harness import assert_bf16_close
    r = Rig([32 * MiB, 4 * MiB])
    try:
        g = si.rng(3, 60)
        n = 100003
        tab, idx, out, src, dst = r.alloc(0, 4 * n), r.alloc(0, 8 * n), r.alloc(0, 4 * n), r.alloc(0, 4 * n), r.alloc(0, 4 * n)
        ws, s_ref, s_out = r.alloc(0, gd.GD_SUM_WORKSPACE), r.alloc(0, 256), r.alloc(0, 256)
        rows, cols = 64, 1024
        x, y, gain = r.alloc(0, 2 * rows * cols), r.alloc(0, 2 * rows * cols), r.alloc(0, 2 * cols)
        M, N, K = 256, 512, 256
        A, B, Cc = r.alloc(0, 2 * M * K), r.alloc(0, 2 * N * K), r.alloc(0, 2 * M * N)
        r.upload(0, tab, si.uniform_f32(g, n))
        r.upload(0, idx, g.integers(0, n, size=n, dtype=np.int64))
        r.upload(0, src, si.uniform_f32(g, n, 0.0, 1.0))
        perm = r.alloc(0, 8 * n)
        r.upload(0, perm, g.permutation(n).astype(np.int64))
        r.upload(0, x, si.f32_to_bf16_bits(si.normal_f32(g, rows * cols)))
        r.upload(0, gain, si.f32_to_bf16_bits(si.uniform_f32(g, cols, 0.5, 1.5)))
        r.upload(0, A, si.f32_to_bf16_bits(si.normal_f32(g, M * K) * np.float32(K ** -0.5)))
        r.upload(0, B, si.f32_to_bf16_bits(si.normal_f32(g, N * K)))
        outputs = [(out, 4 * n), (dst, 4 * n), (s_ref, 4), (s_out, 4), (y, 2 * rows * cols), (Cc, 2 * M * N)]

        def launches(stream):
            r.launch(0, gd.GD_K_GATHER32_I64, gd.gd_args_gather(out, tab, idx, n), stream=stream)
            r.launch(0, gd.GD_K_SCATTER_F32_I64, gd.gd_args_scatter(dst, src, perm, n, 2.0, 0), stream=stream)
            r.launch(0, gd.GD_K_SUM_F32, gd.gd_args_sum(s_ref, src, ws, n), stream=stream)
            gd.gd_sum_f32_noalloc(r.pool, 0, s_out, src, n, stream=stream)
            r.launch(0, gd.GD_K_RMSNORM_BF16, gd.gd_args_rmsnorm(y, x, gain, rows, cols, 1e-6, 0), stream=stream)
            r.launch(0, gd.GD_K_GEMM_BF16, gd.gd_args_gemm(Cc, A, B, M, N, K, 1), stream=stream)

        r.oracle("gather32_i64", 0, out, tab, idx, n)
        r.oracle("scatter_f32_i64", 0, dst, src, perm, 2.0, n)
        r.oracle("sum_f32", 0, s_ref, src, n)
        r.oracle("rmsnorm_bf16", 0, y, x, gain, rows, cols, 1e-6)
        r.oracle("gemm_bf16", 0, Cc, A, B, M, N, K, 1, 0, M, 0, N)
        want_sum = float(r.sim.view(s_ref, np.float32, 1)[0])

        side = torch.cuda.Stream()
        # the allocation-free sum looks its array up on its first call on a device: that call stays outside the capture
        gd.gd_sum_f32_noalloc(r.pool, 0, s_out, src, 16, stream=side.cuda_stream)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            launches(torch.cuda.current_stream().cuda_stream)
        for replay in range(3):
            for (p, nb) in outputs:
                r.dview(p, np.uint8, nb).fill_(0xCD)
            r.dview(ws, np.uint8, gd.GD_SUM_WORKSPACE).fill_(0xCD)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert np.array_equal(r.download(out, np.uint32, n), r.sim.view(out, np.uint32, n)), replay
            assert np.array_equal(r.download(dst, np.uint32, n), r.sim.view(dst, np.uint32, n)), replay
            a, b = r.download(s_ref, np.uint32, 1)[0], r.download(s_out, np.uint32, 1)[0]
            assert a == b, (replay, hex(int(a)), hex(int(b)))
            assert abs(float(np.uint32(a).view(np.float32)) - want_sum) <= FP32_TOL * want_sum
            got_y, want_y = r.download(y, np.uint16, rows * cols), r.sim.view(y, np.uint16, rows * cols)
            assert rel_frobenius(si.bf16_bits_to_f32(got_y), si.bf16_bits_to_f32(want_y)) <= 1e-3 and np.mean(got_y != want_y) < 0.02
            assert_bf16_close(r.download(Cc, np.uint16, M * N), r.sim.view(Cc, np.uint16, M * N), abs_tol=3e-5, what=f"gemm, replay {replay}")
            r.assert_images_equal(skip=outputs + [(ws, gd.GD_SUM_WORKSPACE)], what=f"replay {replay}")
    finally:
        r.close()


def test_one_graph_per_tenant_replayed_on_two_streams_at_once():
    """Each tenant's chain of indexed saxpys (1 % of the offsets out of range, wrapped by the fence into a scratch
    region of the tenant's own partition) is recorded into a graph of its own and the graphs are replayed on the
    tenants' streams at the same time: the tenants' kernels overlap on the chip, and every replay must leave what
    the oracle computes for the chains run one after the other (the tenants share nothing, so the order between
    them cannot matter)."""
    from test_gpu_parity import hazard_free_offsets
    r = Rig([4 * MiB, 4 * MiB])
    try:
        n, rounds, replays = 65536, 20, 3
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        plan, graphs = [], []
        for t in (0, 1):
            g = si.rng(1, 70 + t)
            base, size = r.row(t)
            x, y, off, scratch = (r.alloc(t, 4 * n) for _ in range(4))
            offs, where = hazard_free_offsets(g, n, x, y, scratch, 4 * n, base, size)
            assert len(where) == 655
            r.upload(t, x, si.uniform_f32(g, n))
            r.upload(t, y, si.uniform_f32(g, n))
            r.upload(t, scratch, np.zeros(n, np.float32))
            r.upload(t, off, offs)
            plan.append((t, x, y, off, scratch))
        torch.cuda.synchronize()
        for (t, x, y, off, scratch) in plan:
            cap, graph = torch.cuda.Stream(), torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=cap):
                for _ in range(rounds):
                    r.launch(t, gd.GD_K_SAXPY_IDX, gd.gd_args_saxpy_idx(x, y, off, n, 0.25, 0), stream=torch.cuda.current_stream().cuda_stream)
            graphs.append(graph)
        for replay in range(replays):
            for graph, st in zip(graphs, streams):
                with torch.cuda.stream(st):
                    graph.replay()
            torch.cuda.synchronize()
            for (t, x, y, off, scratch) in plan:
                for _ in range(rounds):
                    r.oracle("saxpy_idx", t, x, y, off, 0.25, n)
                assert r.sim.last[2] >= 3 * 655
            results = [(p, 4 * n) for (t, x, y, off, scratch) in plan for p in (y, scratch)]
            for (p, nb) in results:
                # words equal bit for bit, or saxpy results that differ in the last places (fused multiply-add
                # against fp64 then one rounding, accumulated over the rounds); a wrapped load may have read anything
                got, want = r.download(p, np.float32, n), r.sim.view(p, np.float32, n)
                differ = np.flatnonzero(got.view(np.uint32) != want.view(np.uint32))
                assert np.all(np.isfinite(got[differ])) and np.all(np.isfinite(want[differ])), (replay, hex(p))
                assert np.all(np.abs(got[differ] - want[differ]) <= 4e-6 * np.maximum(1.0, np.abs(want[differ]))), (replay, hex(p))
            # everything but the fp32 results (within tolerance above) byte for byte
            r.assert_images_equal(skip=results, what=f"replay {replay}")
            # both sides go on from the same bits
            for (p, nb) in results:
                r.dview(p, np.uint8, nb).copy_(torch.from_numpy(r.sim.view(p, np.uint8, nb)))
            torch.cuda.synchronize()
    finally:
        r.close()
