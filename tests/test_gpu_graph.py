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
