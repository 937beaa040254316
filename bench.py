#!/usr/bin/env python3
"""Benchmark of the fenced-kernel path on one MI355X.

Headline (`value`): configuration 3 -- 8 tenants, a 16 GiB partition each, one
HIP stream each, fenced STREAM copy + triad on 2^28 fp32 elements per array.
One step = one round: every tenant launches copy then triad on its stream
(16 + 24 = 40 GiB of algorithmic traffic).  All inputs are resident in HBM
before the timed region.  The other four configurations are measured in the
same run and reported under "per_config", each fenced and unfenced (same
kernel, fence off) with the overhead in percent.

Prints ONE JSON line on stdout; progress goes to stderr.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

KiB, MiB, GiB = 1 << 10, 1 << 20, 1 << 30
HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--configs", default="c3,c4,power,c2,c1,c5,modes",
                    help="comma list out of c1..c5 (c3 is the headline), power (GEMM against the chip's power limit), "
                         "modes (the paper's three rules side by side), gatherpolicy (cache-policy bits on random loads) and shapes "
                         "(RMSNorm against the shape, gather against the table size); the last two are not in the default list")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--prewarm-ms", type=float, default=250.0,
                    help="untimed launches in front of every measurement until this much GPU time has passed "
                         "(the shader clock needs tens of milliseconds of load to settle)")
    return ap.parse_args()


# ---------------------------------------------------------------------------------
# device pool plumbing (torch: memory and streams only)
# ---------------------------------------------------------------------------------

class DevPool:
    def __init__(self, torch, gd, sizes, fill=None):
        self.torch, self.gd = torch, gd
        self.sizes = list(sizes)
        biggest, total = max(sizes), sum(sizes)
        self.buf = torch.empty(total + biggest, dtype=torch.uint8, device="cuda")
        raw = self.buf.data_ptr()
        self.base = -(-raw // biggest) * biggest
        self.total = total
        self.dev = self.buf[self.base - raw:self.base - raw + total]
        if fill is not None:
            self.dev.fill_(fill)
        self.pool = gd.gd_pool_create(self.base, total, self.sizes)

    def alloc(self, tenant, nbytes, align=256):
        return self.gd.gd_alloc(self.pool, tenant, nbytes, align)

    def view(self, ptr, nbytes):
        return self.dev[ptr - self.base:ptr - self.base + nbytes]

    def upload(self, tenant, ptr, arr):
        """Checked host-to-device copy: the range check, then the copy."""
        arr = np.ascontiguousarray(arr)
        if self.gd.gd_check_copy(self.pool, tenant, ptr, arr.nbytes) != self.gd.GD_OK:
            raise RuntimeError("copy refused by gd_check_copy")
        self.view(ptr, arr.nbytes).copy_(self.torch.from_numpy(arr.view(np.uint8).reshape(-1)))

    def close(self):
        self.gd.gd_pool_destroy(self.pool)
        self.buf = self.dev = None
        self.torch.cuda.empty_cache()


PREWARM_MS = 250.0


def prewarm(torch, launch):
    """Untimed launches until PREWARM_MS of wall time have passed under load."""
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < PREWARM_MS:
        for _ in range(4):
            launch()
        torch.cuda.synchronize()


def timed_rounds(torch, streams, launch_round, steps, warmup):
    """launch_round(i) enqueues one round on every stream.  Returns seconds for
    `steps` rounds: all streams are released by one event, the clock stops at the
    last stream's end event; bracketed by synchronize on both sides."""
    prewarm(torch, launch_round)
    for _ in range(warmup):
        launch_round()
    torch.cuda.synchronize()
    go = torch.cuda.Event(enable_timing=True)
    ends = [torch.cuda.Event(enable_timing=True) for _ in streams]
    t0 = time.perf_counter()
    go.record()
    for s in streams:
        s.wait_event(go)
    for _ in range(steps):
        launch_round()
    for s, e in zip(streams, ends):
        e.record(s)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per_stream = [go.elapsed_time(e) * 1e-3 for e in ends]
    timed_rounds.per_stream = per_stream           # seconds from the release to each stream's end event
    return max(per_stream), wall


def solo_avg_seconds(torch, stream, launch, reps, warmup=2):
    """Average duration of one launch, back to back on one stream, by HIP events
    recorded on that stream."""
    prewarm(torch, launch)
    for _ in range(warmup):
        launch()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(stream)
    for _ in range(reps):
        launch()
    b.record(stream)
    torch.cuda.synchronize()
    return a.elapsed_time(b) * 1e-3 / reps


def pct_overhead(fenced_rate, unfenced_rate):
    return round(100.0 * (unfenced_rate / fenced_rate - 1.0), 2) if fenced_rate else None


# ---------------------------------------------------------------------------------
# configuration 3 (headline): 8 tenants x 16 GiB, copy + triad on 8 streams
# ---------------------------------------------------------------------------------

def run_c3(torch, gd, si, args):
    n = 1 << 28
    tenants = 8
    log(f"[c3] carving {tenants} x 16 GiB and uploading seeded inputs")
    dp = DevPool(torch, gd, [16 * GiB] * tenants)
    streams = [torch.cuda.Stream() for _ in range(tenants)]
    host = np.empty(n, np.float32)
    plan = []
    for t in range(tenants):
        a, b, c = (dp.alloc(t, 4 * n) for _ in range(3))
        for part, ptr in ((1, b), (2, c)):
            si.fill_chunked(host, 3, t + 100 * part, "uniform", threads=16)
            dp.upload(t, ptr, host)
        s = float(si.uniform_f32(si.rng(3, t), 1)[0])
        plan.append((t, a, b, c, s))
    torch.cuda.synchronize()
    del host

    def round_of(mode, active=tenants):
        def go():
            for (t, a, b, c, s), st in zip(plan[:active], streams):
                gd.gd_launch_fenced(dp.pool, t, gd.GD_K_COPY, gd.gd_args_copy(a, b, n), stream=st.cuda_stream, mode=mode)
                gd.gd_launch_fenced(dp.pool, t, gd.GD_K_TRIAD, gd.gd_args_triad(a, b, c, n, s, 0), stream=st.cuda_stream, mode=mode)
        return go

    bytes_round = tenants * (8 + 12) * n
    res = {}
    for name, mode in (("fenced", gd.GD_FENCE_BITWISE), ("unfenced", gd.GD_FENCE_NONE)):
        dev, wall = timed_rounds(torch, streams, round_of(mode), args.steps, args.warmup)
        res[name] = {"seconds": dev, "wall_seconds": wall, "GBps": bytes_round * args.steps / dev / 1e9}
        log(f"[c3] {name}: {res[name]['GBps']:.1f} GB/s aggregate over {tenants} streams ({dev / args.steps * 1e3:.3f} ms/round)")

    # the same round with 1, 2 and 4 of the tenants active (co-location, the paper's Section 7.1 setting): aggregate rate
    by_tenants = {}
    for active in (1, 2, 4):
        row = {}
        for name, mode in (("fenced", gd.GD_FENCE_BITWISE), ("unfenced", gd.GD_FENCE_NONE)):
            dev, _ = timed_rounds(torch, streams[:active], round_of(mode, active), max(3, args.steps // 2), 1)
            row[name + "_GBps"] = active * (8 + 12) * n * max(3, args.steps // 2) / dev / 1e9
        row["overhead_pct"] = pct_overhead(row["fenced_GBps"], row["unfenced_GBps"])
        by_tenants[str(active)] = row
        log(f"[c3] {active} tenant(s) active: fenced {row['fenced_GBps']:.1f} / unfenced {row['unfenced_GBps']:.1f} GB/s aggregate")
    by_tenants[str(tenants)] = {"fenced_GBps": res["fenced"]["GBps"], "unfenced_GBps": res["unfenced"]["GBps"],
                                "overhead_pct": pct_overhead(res["fenced"]["GBps"], res["unfenced"]["GBps"])}

    # each kernel alone on tenant 0's stream: the per-launch figures of the roofline
    t, a, b, c, s = plan[0]
    st = streams[0]
    solo = {}
    for kname, kid, kargs, nbytes in (("copy", gd.GD_K_COPY, gd.gd_args_copy(a, b, n), 8 * n),
                                      ("triad", gd.GD_K_TRIAD, gd.gd_args_triad(a, b, c, n, s, 0), 12 * n)):
        for name, mode in (("fenced", gd.GD_FENCE_BITWISE), ("unfenced", gd.GD_FENCE_NONE)):
            sec = solo_avg_seconds(torch, st, lambda: gd.gd_launch_fenced(dp.pool, t, kid, kargs, stream=st.cuda_stream, mode=mode), args.steps)
            solo[f"{kname}_{name}"] = {"avg_launch_ms": sec * 1e3, "GBps": nbytes / sec / 1e9}
            log(f"[c3] {kname} {name} alone: {nbytes / sec / 1e9:.1f} GB/s ({sec * 1e3:.3f} ms/launch)")
    dp.close()
    return {
        "workload": "8 tenants x 16 GiB partitions, 8 streams, fp32 copy + triad, 2^28 elements per array",
        "bytes_per_round": bytes_round,
        "fenced_GBps": res["fenced"]["GBps"], "unfenced_GBps": res["unfenced"]["GBps"],
        "overhead_pct": pct_overhead(res["fenced"]["GBps"], res["unfenced"]["GBps"]),
        "frac_of_hbm_peak": res["fenced"]["GBps"] / HBM_PEAK_GBPS,
        "ms_per_round_fenced": res["fenced"]["seconds"] / args.steps * 1e3,
        "wall_seconds_fenced": res["fenced"]["wall_seconds"],
        "solo": solo,
        "aggregate_by_active_tenants": by_tenants,
        "triad_bytes_per_launch": 12 * n,
    }


# ---------------------------------------------------------------------------------
# configuration 4: bf16 GEMM 8192^3 in a 4 GiB partition
# ---------------------------------------------------------------------------------

def run_c4(torch, gd, si, args):
    M = N = K = 8192
    log("[c4] GEMM 8192^3 bf16")
    dp = DevPool(torch, gd, [4 * GiB])
    A, B, Cc = (dp.alloc(0, 2 * M * K) for _ in range(3))
    host = np.empty(M * K, np.float32)
    si.fill_chunked(host, 4, 1, "normal", threads=16)
    dp.upload(0, A, si.f32_to_bf16_bits(host * np.float32(K ** -0.5)))
    si.fill_chunked(host, 4, 2, "normal", threads=16)
    dp.upload(0, B, si.f32_to_bf16_bits(host))
    del host
    st = torch.cuda.Stream()
    kargs = gd.gd_args_gemm(Cc, A, B, M, N, K, 1)
    flop = 2.0 * M * N * K
    out = {"workload": "1 tenant, 4 GiB partition, C = A*B, M=N=K=8192, bf16 in/out, fp32 accumulate, B stored N x K", "flop": flop}
    for name, mode in (("fenced", gd.GD_FENCE_BITWISE), ("unfenced", gd.GD_FENCE_NONE)):
        sec = solo_avg_seconds(torch, st, lambda: gd.gd_launch_fenced(dp.pool, 0, gd.GD_K_GEMM_BF16, kargs, stream=st.cuda_stream, mode=mode), args.steps)
        out[f"{name}_TFLOPs"] = flop / sec / 1e12
        out[f"{name}_ms"] = sec * 1e3
        log(f"[c4] {name}: {flop / sec / 1e12:.1f} TFLOP/s ({sec * 1e3:.3f} ms)")
    out["overhead_pct"] = pct_overhead(out["fenced_TFLOPs"], out["unfenced_TFLOPs"])
    out["frac_of_mfma_peak"] = out["fenced_TFLOPs"] / MFMA_BF16_PEAK_TFLOPS
    dp.close()
    return out


# ---------------------------------------------------------------------------------
# configuration 2: gather then scatter, 2^26 elements, 0.1 % of indices out of bounds
# ---------------------------------------------------------------------------------

def run_c2(torch, gd, si, args):
    n = tab_n = 1 << 26
    log("[c2] gather/scatter 2^26")
    dp = DevPool(torch, gd, [1 * GiB, 1 * GiB])
    canary = si.address_canary(1 << 20)
    nb_base, nb_size, _ = gd.gd_partition_info(dp.pool, 1)
    for k in range(0, nb_size, canary.nbytes):
        dp.upload(1, nb_base + k, canary)
    tab, idx, out = dp.alloc(0, 4 * tab_n), dp.alloc(0, 8 * n), dp.alloc(0, 4 * n)
    host = np.empty(tab_n, np.float32)
    si.fill_chunked(host, 2, 1, "normal", threads=16)
    dp.upload(0, tab, host)
    del host
    ix, where = si.c2_indices(si.rng(2, 0), n, tab_n)
    dp.upload(0, idx, ix)
    st = torch.cuda.Stream()
    res = {"workload": "1 tenant, 1 GiB partition, fp32 table 2^26, int64 indices 2^26 (0.1 % in [2^26, 2^30)), gather then scatter; neighbour partition holds a canary",
           "bytes_per_launch": 16 * n}
    g_args, s_args = gd.gd_args_gather(out, tab, idx, n), gd.gd_args_scatter(tab, out, idx, n, -1.0, 0)
    for kname, kid, kargs in (("gather", gd.GD_K_GATHER32_I64, g_args), ("scatter", gd.GD_K_SCATTER_F32_I64, s_args)):
        # the unfenced build may only see in-bounds indices
        for name, mode in (("fenced", gd.GD_FENCE_BITWISE), ("fenced_inbounds", gd.GD_FENCE_BITWISE), ("unfenced_inbounds", gd.GD_FENCE_NONE)):
            if name == "fenced_inbounds":
                ix[where] = ix[(where + 1) % n] % tab_n
                dp.upload(0, idx, ix)
            sec = solo_avg_seconds(torch, st, lambda: gd.gd_launch_fenced(dp.pool, 0, kid, kargs, stream=st.cuda_stream, mode=mode), max(3, args.steps // 2))
            res[f"{kname}_{name}_GBps"] = 16 * n / sec / 1e9
            log(f"[c2] {kname} {name}: {16 * n / sec / 1e9:.1f} GB/s ({sec * 1e3:.3f} ms)")
        res[f"{kname}_overhead_pct"] = pct_overhead(res[f"{kname}_fenced_inbounds_GBps"], res[f"{kname}_unfenced_inbounds_GBps"])
        ix, where = si.c2_indices(si.rng(2, 0), n, tab_n)
        dp.upload(0, idx, ix)
    torch.cuda.synchronize()
    want = torch.from_numpy(canary.view(np.int64)).cuda()
    got = dp.view(nb_base, nb_size).view(torch.int64).reshape(-1, want.numel())
    res["canary_intact"] = bool((got == want).all().item())
    dp.close()
    return res


# ---------------------------------------------------------------------------------
# configuration 1: two tenants, 4 MiB partitions, indexed saxpy, 1 % offsets out of range
# ---------------------------------------------------------------------------------

def run_c1(torch, gd, si, args):
    n = 262144
    log("[c1] indexed saxpy, 2 tenants")
    dp = DevPool(torch, gd, [4 * MiB, 4 * MiB], fill=0xA5)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    plans = {}
    for literal in (True, False):
        plan = []
        for t in range(2):
            base, size, _ = gd.gd_partition_info(dp.pool, t)
            g = si.rng(1, t)
            if literal:
                x, y, off = (dp.alloc(t, 4 * n) for _ in range(3))
            else:
                x, y, off = plans[True][t][1:4]
            offs, where = si.c1_offsets(g, n, y, base, size)
            if not literal:
                offs = np.arange(n, dtype=np.int32)
            plan.append((t, x, y, off, offs, float(si.uniform_f32(g, 1)[0])))
        plans[literal] = plan
    launches = 1000
    literal_launches = 50
    res = {"workload": "2 tenants x 4 MiB partitions, 2 streams, fp32 y[o]=a*x[o]+y[o], n=262144, 1 % of offsets out of range",
           "bytes_per_tenant_launch": 16 * n, "launches_per_stream": launches,
           "note": "every wrapped store of the literal run lands in the tenant's own partition, a quarter of them on its "
                   "offset array, so repeated launches feed on their own damage; the literal figure is therefore taken "
                   f"over the first {literal_launches} launches after a fresh upload, the overhead from the in-bounds pair"}

    def upload(plan):
        g = si.rng(1, 50)
        for (t, x, y, off, offs, alpha) in plan:
            dp.upload(t, x, si.uniform_f32(g, n))
            dp.upload(t, y, np.zeros(n, np.float32))
            dp.upload(t, off, offs)

    def round_of(plan, mode):
        def go():
            for (t, x, y, off, offs, alpha), st in zip(plan, streams):
                gd.gd_launch_fenced(dp.pool, t, gd.GD_K_SAXPY_IDX, gd.gd_args_saxpy_idx(x, y, off, n, alpha * 1e-3, 0), stream=st.cuda_stream, mode=mode)
        return go

    for name, mode in (("fenced_inbounds", gd.GD_FENCE_BITWISE), ("unfenced_inbounds", gd.GD_FENCE_NONE)):
        upload(plans[False])
        dev, _ = timed_rounds(torch, streams, round_of(plans[False], mode), launches, 20)
        res[f"{name}_GBps"] = 2 * 16 * n * launches / dev / 1e9
        res[f"{name}_us_per_round"] = dev / launches * 1e6
        log(f"[c1] {name}: {res[f'{name}_GBps']:.1f} GB/s effective ({dev / launches * 1e6:.2f} us per 2-tenant round)")
    # The same in-bounds rounds recorded once into a HIP graph (gd_launch_fenced allocates and
    # synchronises nothing, so it can be captured) and replayed: what a launch-bound caller gains.
    def graph_us_per_round(mode, rounds=200, replays=5):
        cap, side = torch.cuda.Stream(), torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        plan = plans[False]
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=cap):
            cur = torch.cuda.current_stream()
            side.wait_stream(cur)
            for _ in range(rounds):
                for (t, x, y, off, offs, alpha), st in zip(plan, (cur, side)):
                    gd.gd_launch_fenced(dp.pool, t, gd.GD_K_SAXPY_IDX, gd.gd_args_saxpy_idx(x, y, off, n, alpha * 1e-3, 0), stream=st.cuda_stream, mode=mode)
            cur.wait_stream(side)
        for _ in range(2):
            graph.replay()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(replays):
            graph.replay()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / (rounds * replays)

    # One graph per tenant, replayed on the tenant's own stream: each tenant's launches follow one another on the
    # GPU without the host, and the two tenants' kernels can overlap (they fill a quarter of the chip each).
    def graphs_per_tenant_us_per_round(mode, rounds=200, replays=5):
        graphs = []
        torch.cuda.synchronize()
        for (t, x, y, off, offs, alpha) in plans[False]:
            cap, graph = torch.cuda.Stream(), torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=cap):
                cur = torch.cuda.current_stream()
                for _ in range(rounds):
                    gd.gd_launch_fenced(dp.pool, t, gd.GD_K_SAXPY_IDX, gd.gd_args_saxpy_idx(x, y, off, n, alpha * 1e-3, 0), stream=cur.cuda_stream, mode=mode)
            graphs.append(graph)

        def replay_all():
            for graph, st in zip(graphs, streams):
                with torch.cuda.stream(st):
                    graph.replay()
        for _ in range(2):
            replay_all()
        torch.cuda.synchronize()
        go = torch.cuda.Event(enable_timing=True)
        ends = [torch.cuda.Event(enable_timing=True) for _ in streams]
        go.record()
        for st in streams:
            st.wait_event(go)
        for _ in range(replays):
            replay_all()
        for st, e in zip(streams, ends):
            e.record(st)
        torch.cuda.synchronize()
        return max(go.elapsed_time(e) for e in ends) * 1e3 / (rounds * replays)

    try:
        upload(plans[False])
        res["graph_per_tenant_fenced_inbounds_us_per_round"] = graphs_per_tenant_us_per_round(gd.GD_FENCE_BITWISE)
        res["graph_per_tenant_unfenced_inbounds_us_per_round"] = graphs_per_tenant_us_per_round(gd.GD_FENCE_NONE)
        log(f"[c1] one graph per tenant, replayed on two streams: fenced {res['graph_per_tenant_fenced_inbounds_us_per_round']:.2f} / unfenced "
            f"{res['graph_per_tenant_unfenced_inbounds_us_per_round']:.2f} us per 2-tenant round")
    except Exception as ex:                       # informational figure: never lose the run over it
        res["graph_per_tenant_error"] = repr(ex)
        log(f"[c1] per-tenant graph replay failed: {ex!r}")
        torch.cuda.synchronize()

    try:
        upload(plans[False])
        res["graph_fenced_inbounds_us_per_round"] = graph_us_per_round(gd.GD_FENCE_BITWISE)
        res["graph_unfenced_inbounds_us_per_round"] = graph_us_per_round(gd.GD_FENCE_NONE)
        log(f"[c1] graph replay: fenced {res['graph_fenced_inbounds_us_per_round']:.2f} / unfenced "
            f"{res['graph_unfenced_inbounds_us_per_round']:.2f} us per 2-tenant round")
    except Exception as ex:                       # informational figure: never lose the run over it
        res["graph_error"] = repr(ex)
        log(f"[c1] graph replay failed: {ex!r}")
        torch.cuda.synchronize()

    # literal offsets: the clock is warm from the runs above; fresh inputs, no further warm-up
    global PREWARM_MS
    keep, PREWARM_MS = PREWARM_MS, 0.0
    upload(plans[True])
    torch.cuda.synchronize()
    dev, _ = timed_rounds(torch, streams, round_of(plans[True], gd.GD_FENCE_BITWISE), literal_launches, 0)
    PREWARM_MS = keep
    res["fenced_GBps"] = 2 * 16 * n * literal_launches / dev / 1e9
    res["fenced_us_per_round"] = dev / literal_launches * 1e6
    log(f"[c1] fenced, literal offsets, first {literal_launches} launches: {res['fenced_GBps']:.1f} GB/s effective ({dev / literal_launches * 1e6:.2f} us per round)")
    res["overhead_pct"] = pct_overhead(res["fenced_inbounds_GBps"], res["unfenced_inbounds_GBps"])
    dp.close()
    return res


# ---------------------------------------------------------------------------------
# configuration 5: 16 tenants, mixed partition sizes, sum / RMSNorm / int32 gather, re-carve
# ---------------------------------------------------------------------------------

def run_c5(torch, gd, si, args):
    g = si.rng(5, 0)
    sizes = si.c5_partition_sizes(g, 16, budget=128 * GiB)
    log(f"[c5] 16 tenants, sizes (MiB): {[s // MiB for s in sizes]}")
    dp = DevPool(torch, gd, sizes)
    streams = [torch.cuda.Stream() for _ in sizes]
    n_sum, rows, cols, n_g = 1 << 27, 4096, 8192, 1 << 24

    def setup(t, kind):
        gt = si.rng(5, t + 1)
        if kind == "sum":
            src, ws, out = dp.alloc(t, 4 * n_sum), dp.alloc(t, gd.GD_SUM_WORKSPACE), dp.alloc(t, 256)
            host = np.empty(n_sum, np.float32)
            si.fill_chunked(host, 5, t + 1, "uniform", 0.0, 1.0, threads=16)
            dp.upload(t, src, host)
            return gd.GD_K_SUM_F32, gd.gd_args_sum(out, src, ws, n_sum), 4 * n_sum, [src, ws, out]
        if kind == "rmsnorm":
            x, y, gain = dp.alloc(t, 2 * rows * cols), dp.alloc(t, 2 * rows * cols), dp.alloc(t, 2 * cols)
            dp.upload(t, x, si.f32_to_bf16_bits(si.normal_f32(gt, rows * cols)))
            dp.upload(t, gain, si.f32_to_bf16_bits(si.uniform_f32(gt, cols, 0.5, 1.5)))
            return gd.GD_K_RMSNORM_BF16, gd.gd_args_rmsnorm(y, x, gain, rows, cols, 1e-6, 0), 4 * rows * cols, [x, y, gain]
        tab, idx, out = dp.alloc(t, 4 * n_g), dp.alloc(t, 4 * n_g), dp.alloc(t, 4 * n_g)
        dp.upload(t, tab, gt.integers(-2**31, 2**31, size=n_g, dtype=np.int64).astype(np.int32))
        dp.upload(t, idx, si.c5_indices_i32(gt, n_g, n_g)[0])
        return gd.GD_K_GATHER32_I32, gd.gd_args_gather(out, tab, idx, n_g), 12 * n_g, [tab, idx, out]

    kinds = ["sum", "rmsnorm", "gather"]
    work = {}
    k = 0
    for t, s in enumerate(sizes):
        kind = kinds[k % 3]
        if kind == "sum" and s < GiB:
            kind = "rmsnorm" if (k // 3) % 2 == 0 else "gather"
        k += 1
        work[t] = (kind,) + setup(t, kind)
    if not any(w[0] == "sum" for w in work.values()):
        raise RuntimeError("no tenant large enough for the reduction")
    torch.cuda.synchronize()

    res = {"workload": "16 tenants, pow2 partitions in [256 MiB, 8 GiB], 16 streams: fp32 sum 2^27, bf16 RMSNorm 4096x8192, int32 gather 2^24 (0.5 % out of bounds); 4 tenants re-carved mid-run",
           "partition_MiB": [s // MiB for s in sizes], "assignment": [work[t][0] for t in range(16)]}
    # each kernel alone
    for kind in kinds:
        t = next(t for t in work if work[t][0] == kind)
        _, kid, kargs, nbytes, _ = work[t]
        for name, mode in (("fenced", gd.GD_FENCE_BITWISE), ("unfenced", gd.GD_FENCE_NONE)):
            if kind == "gather" and mode == gd.GD_FENCE_NONE:
                dp.upload(t, kargs.idx, np.abs(si.c5_indices_i32(si.rng(5, t + 1), n_g, n_g)[0]) % n_g)
            sec = solo_avg_seconds(torch, streams[t], lambda: gd.gd_launch_fenced(dp.pool, t, kid, kargs, stream=streams[t].cuda_stream, mode=mode), args.steps)
            res[f"{kind}_{name}_GBps"] = nbytes / sec / 1e9
            log(f"[c5] {kind} {name} alone: {nbytes / sec / 1e9:.1f} GB/s ({sec * 1e6:.1f} us)")
        if kind == "gather":
            sec = solo_avg_seconds(torch, streams[t], lambda: gd.gd_launch_fenced(dp.pool, t, kid, kargs, stream=streams[t].cuda_stream, mode=gd.GD_FENCE_BITWISE), args.steps)
            res["gather_fenced_inbounds_GBps"] = nbytes / sec / 1e9
            res["gather_overhead_pct"] = pct_overhead(res["gather_fenced_inbounds_GBps"], res["gather_unfenced_GBps"])
            dp.upload(t, kargs.idx, si.c5_indices_i32(si.rng(5, t + 1), n_g, n_g)[0])
        else:
            res[f"{kind}_overhead_pct"] = pct_overhead(res[f"{kind}_fenced_GBps"], res[f"{kind}_unfenced_GBps"])

    def mixed_round():
        for t, (kind, kid, kargs, nbytes, _) in work.items():
            gd.gd_launch_fenced(dp.pool, t, kid, kargs, stream=streams[t].cuda_stream, mode=gd.GD_FENCE_BITWISE)

    def breakdown(dev):
        """Per kind of kernel in the mixed rounds: tenants, their share of the bytes, and when their
        streams finished (all streams start together, so a kind that ends late is what the round waits for)."""
        out = {}
        for kind in kinds:
            ts = [t for t in work if work[t][0] == kind]
            if not ts:
                continue
            end = [timed_rounds.per_stream[t] for t in ts]
            nbytes = sum(work[t][3] for t in ts) * args.steps
            out[kind] = {"tenants": len(ts), "bytes_share": round(sum(work[t][3] for t in ts) / sum(w[3] for w in work.values()), 3),
                         "last_stream_done_at_frac_of_round": round(max(end) / dev, 3),
                         "GBps_until_its_last_stream_ends": round(nbytes / max(end) / 1e9, 1)}
        return out

    bytes_round = sum(w[3] for w in work.values())
    dev, _ = timed_rounds(torch, streams, mixed_round, args.steps, args.warmup)
    res["mixed_fenced_GBps_before_recarve"] = bytes_round * args.steps / dev / 1e9
    res["mixed_breakdown_before_recarve"] = breakdown(dev)
    # what the same launches would take one after the other at their solo rates: the mixed round is bound by the
    # gathers (line traffic, see the solo figures), which take most of the time while moving a small share of the bytes
    res["mixed_serial_estimate_GBps"] = round(bytes_round / sum(w[3] / (res[f"{w[0]}_fenced_GBps"] * 1e9) for w in work.values()) / 1e9, 1)

    # re-carve: four tenants free everything, detach, and come back with another size
    t0 = time.perf_counter()
    movers = [int(t) for t in g.choice(16, size=4, replace=False)]
    for t in movers:
        for p in work[t][4]:
            gd.gd_free(dp.pool, t, p)
        gd.gd_tenant_detach(dp.pool, t)
    resized = sorted(((sizes[t] // 2 if sizes[t] > 512 * MiB else sizes[t] * 2), t) for t in movers)[::-1]
    for new_size, t in resized:
        for trial in (new_size, sizes[t], sizes[t] // 2):
            try:
                nt = gd.gd_tenant_attach(dp.pool, trial)
                new_size = trial
                break
            except gd.GuardianError as e:
                if e.status != gd.GD_ENOMEM:
                    raise
        else:
            raise RuntimeError("re-carve: no room for a returning tenant")
        kind = "rmsnorm" if new_size < GiB or work[t][0] != "sum" else "sum"
        del work[t]
        work[nt] = (kind,) + setup(nt, kind)
    res["recarve_host_ms"] = (time.perf_counter() - t0) * 1e3
    torch.cuda.synchronize()
    bytes_round = sum(w[3] for w in work.values())
    dev, _ = timed_rounds(torch, streams, mixed_round, args.steps, args.warmup)
    res["mixed_fenced_GBps_after_recarve"] = bytes_round * args.steps / dev / 1e9
    res["mixed_breakdown_after_recarve"] = breakdown(dev)
    res["assignment_after_recarve"] = {int(t): work[t][0] for t in sorted(work)}
    log(f"[c5] mixed 16-stream rounds: {res['mixed_fenced_GBps_before_recarve']:.1f} GB/s before, {res['mixed_fenced_GBps_after_recarve']:.1f} GB/s after the re-carve")
    dp.close()
    return res


# ---------------------------------------------------------------------------------
# the GEMM against the power limit: matrix instructions alone, and the GEMM on zero operands
# ---------------------------------------------------------------------------------

class PowerSampler:
    """Socket power (W) and shader clock (MHz) of GPU 0 from the amdgpu hwmon files, sampled by a thread."""

    def __init__(self):
        import glob
        def first(pattern):
            hits = sorted(glob.glob(pattern))
            return hits[0] if hits else None
        self.power = first("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input") or \
            first("/sys/class/drm/card*/device/hwmon/hwmon*/power1_average")
        self.clock = first("/sys/class/drm/card*/device/hwmon/hwmon*/freq1_input")
        self.dpm = None if self.clock else first("/sys/class/drm/card*/device/pp_dpm_sclk")   # "1: 1870Mhz *" marks the current level

    @staticmethod
    def _read(path):
        try:
            with open(path) as f:
                return float(f.read().split()[0])
        except (OSError, ValueError, IndexError):
            return None

    def run(self, seconds, skip):
        """Sample for `seconds`, drop what was read in the first `skip` seconds; returns (watts, MHz) means or None."""
        t0 = time.perf_counter()
        watts, mhz = [], []
        while time.perf_counter() - t0 < seconds:
            if time.perf_counter() - t0 >= skip:
                w = self._read(self.power) if self.power else None
                c = self._read(self.clock) if self.clock else None
                if w is not None:
                    watts.append(w * 1e-6)
                if c is not None:
                    mhz.append(c * 1e-6)
                elif self.dpm:
                    try:
                        cur = [ln for ln in open(self.dpm).read().splitlines() if ln.rstrip().endswith("*")]
                        mhz.append(float(cur[0].split(":")[1].lower().replace("mhz", "").replace("*", "").strip()))
                    except (OSError, ValueError, IndexError):
                        pass
            time.sleep(0.01)
        mean = lambda v: round(sum(v) / len(v), 1) if v else None
        return mean(watts), mean(mhz)


def run_power(torch, gd, si, args):
    """Is the GEMM held back by the kernel or by the chip's power limit?  Same instrument for five loops of about
    a second each: the matrix instructions alone (operands in registers) on N(0,1) and on zero data, and the GEMM
    on N(0,1) (fenced, unfenced) and on zero operands.  Rate from HIP events over the whole loop, power and clock
    from the driver's hwmon files while it runs."""
    import threading
    log("[power] matrix pipe alone vs GEMM, N(0,1) vs zero operands")
    M = N = K = 8192
    dp = DevPool(torch, gd, [4 * GiB])
    A, B, Cc = (dp.alloc(0, 2 * M * K) for _ in range(3))
    host = np.empty(M * K, np.float32)
    si.fill_chunked(host, 4, 1, "normal", threads=16)
    a_bits = si.f32_to_bf16_bits(host * np.float32(K ** -0.5))
    si.fill_chunked(host, 4, 2, "normal", threads=16)
    b_bits = si.f32_to_bf16_bits(host)
    del host
    st = torch.cuda.Stream()
    blocks = 1024
    ops = torch.empty(16 * 256 * 8, dtype=torch.int16, device="cuda")
    sums = torch.empty(blocks * 256, dtype=torch.float32, device="cuda")
    sampler = PowerSampler()
    res = {"workload": "8192^3 bf16 GEMM and a loop of its matrix instructions alone (1024 workgroups x 4 wavefronts, operands in registers), ~1 s each",
           "power_file": sampler.power, "clock_file": sampler.clock or sampler.dpm, "power_cap_note": "hwmon power1_input is the socket power the driver reports"}

    def loop(label, launch, flop_per_launch, seconds=1.2):
        prewarm(torch, launch)
        n = 0
        got = {}
        th = threading.Thread(target=lambda: got.update(zip(("watts", "mhz"), sampler.run(seconds, 0.3))))
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        th.start()
        a.record(st)
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < seconds:
            for _ in range(20):
                launch()
            n += 20
            torch.cuda.synchronize()
        b.record(st)
        torch.cuda.synchronize()
        th.join()
        tf = flop_per_launch * n / (a.elapsed_time(b) * 1e-3) / 1e12
        res[label] = {"TFLOPs": round(tf, 1), "socket_watts": got.get("watts"), "shader_MHz": got.get("mhz"),
                      "frac_of_mfma_peak": round(tf / MFMA_BF16_PEAK_TFLOPS, 4)}
        log(f"[power] {label}: {tf:.1f} TFLOP/s, {got.get('watts')} W, {got.get('mhz')} MHz")

    iters = 2048
    probe_flop = blocks * 4 * iters * float(1 << 20)
    frag = np.concatenate([a_bits[: 8 * 256 * 8], b_bits[: 8 * 256 * 8]])
    ops.copy_(torch.from_numpy(frag.view(np.int16)))
    loop("mfma_only_normal_operands", lambda: gd.gd_probe_mfma(ops.data_ptr(), sums.data_ptr(), blocks, iters, stream=st.cuda_stream), probe_flop)
    ops.zero_()
    loop("mfma_only_zero_operands", lambda: gd.gd_probe_mfma(ops.data_ptr(), sums.data_ptr(), blocks, iters, stream=st.cuda_stream), probe_flop)
    kargs = gd.gd_args_gemm(Cc, A, B, M, N, K, 1)
    flop = 2.0 * M * N * K
    dp.upload(0, A, a_bits)
    dp.upload(0, B, b_bits)
    for name, mode in (("gemm_fenced_normal_operands", gd.GD_FENCE_BITWISE), ("gemm_unfenced_normal_operands", gd.GD_FENCE_NONE)):
        loop(name, lambda: gd.gd_launch_fenced(dp.pool, 0, gd.GD_K_GEMM_BF16, kargs, stream=st.cuda_stream, mode=mode), flop)
    # context only, not part of the path: the vendor library's kernel for the same product on the same operands under
    # the same power cap (torch.matmul of the two bf16 matrices where they lie in the pool; B is stored N x K)
    try:
        ta = dp.view(A, 2 * M * K).view(torch.bfloat16).view(M, K)
        tb = dp.view(B, 2 * M * K).view(torch.bfloat16).view(N, K)
        tc = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")

        def vendor():
            with torch.cuda.stream(st):
                torch.matmul(ta, tb.t(), out=tc)
        loop("vendor_library_gemm_normal_operands", vendor, flop)
        del ta, tb, tc
    except Exception as ex:                       # context figure: never lose the run over it
        res["vendor_library_error"] = repr(ex)
        torch.cuda.synchronize()
    dp.view(A, 2 * M * K).zero_()
    dp.view(B, 2 * M * K).zero_()
    loop("gemm_fenced_zero_operands", lambda: gd.gd_launch_fenced(dp.pool, 0, gd.GD_K_GEMM_BF16, kargs, stream=st.cuda_stream, mode=gd.GD_FENCE_BITWISE), flop)
    g, m = res["gemm_fenced_normal_operands"]["TFLOPs"], res["mfma_only_normal_operands"]["TFLOPs"]
    res["gemm_frac_of_mfma_only_rate_same_data"] = round(g / m, 4) if m else None
    dp.close()
    return res


# ---------------------------------------------------------------------------------
# random 4-byte loads under every cache-policy combination (not in the default list)
# ---------------------------------------------------------------------------------

def run_gatherpolicy(torch, gd, si, args):
    """Configuration 2's gather (table 2^26 fp32, 2^26 int64 indices, in bounds) with the table load carrying each
    combination of the sc0 / sc1 / nt bits.  Run under `rocprofv3 --pmc FETCH_SIZE` to read the bytes fetched past
    the L2 per variant; the times here show whether any combination helps."""
    n = tab_n = 1 << 26
    log("[gatherpolicy] random 4-byte loads from a 256 MiB table, 8 cache-policy combinations")
    tab = torch.empty(tab_n, dtype=torch.float32, device="cuda").normal_()
    idx = torch.from_numpy(si.rng(2, 0).integers(0, tab_n, size=n, dtype=np.int64)).cuda()
    out = torch.empty(n, dtype=torch.float32, device="cuda")
    st = torch.cuda.Stream()
    names = ("none", "sc0", "sc1", "sc0 sc1", "nt", "sc0 nt", "sc1 nt", "sc0 sc1 nt")
    res = {"workload": "unfenced gather of 2^26 fp32 values through 2^26 uniform int64 indices over a 256 MiB table, per cache-policy bits on the table load"}
    for p, name in enumerate(names):
        sec = solo_avg_seconds(torch, st, lambda: gd.gd_probe_gather_policy(out.data_ptr(), tab.data_ptr(), idx.data_ptr(), n, p, stream=st.cuda_stream), max(3, args.steps // 2))
        res[name] = {"ms": round(sec * 1e3, 4), "GBps_algorithmic": round(16 * n / sec / 1e9, 1)}
        log(f"[gatherpolicy] {name:11s}: {sec * 1e3:.3f} ms, {16 * n / sec / 1e9:.1f} GB/s algorithmic")
    assert torch.equal(out, tab[idx])
    return res


def run_shapes(torch, gd, si, args):
    """Not part of the default run: RMSNorm over matrices of several shapes (cache resident and not, rows of up to
    32768 columns) and the int64 gather against the size of its table, fenced (bitwise) and unfenced."""
    log("[shapes] RMSNorm against the shape, gather against the table size")
    dp = DevPool(torch, gd, [4 * GiB])
    st = torch.cuda.Stream()
    res = {"workload": "1 tenant, 4 GiB partition, all accesses in bounds", "rmsnorm": {}, "gather_i64_2^26_indices": {}}
    both = (("fenced", gd.GD_FENCE_BITWISE), ("unfenced", gd.GD_FENCE_NONE))
    for rows, cols in ((4096, 8192), (16384, 8192), (8192, 4096), (32768, 4096), (2730, 12288), (2048, 16384), (1024, 32768), (4096, 8200), (4096, 8190)):
        nbytes = 2 * rows * cols
        x, y, gain = dp.alloc(0, nbytes), dp.alloc(0, nbytes), dp.alloc(0, 2 * cols)
        dp.view(x, nbytes).view(torch.bfloat16).normal_()
        dp.view(gain, 2 * cols).view(torch.bfloat16).uniform_(0.5, 1.5)
        kargs = gd.gd_args_rmsnorm(y, x, gain, rows, cols, 1e-6, 0)
        row = {}
        for name, mode in both:
            sec = solo_avg_seconds(torch, st, lambda: gd.gd_launch_fenced(dp.pool, 0, gd.GD_K_RMSNORM_BF16, kargs, stream=st.cuda_stream, mode=mode), max(10, args.steps))
            row[name + "_GBps"], row[name + "_us"] = round(2 * nbytes / sec / 1e9, 1), round(sec * 1e6, 2)
        res["rmsnorm"][f"{rows}x{cols}"] = row
        log(f"[shapes] rmsnorm {rows} x {cols}: fenced {row['fenced_GBps']} / unfenced {row['unfenced_GBps']} GB/s")
        for ptr in (x, y, gain):
            gd.gd_free(dp.pool, 0, ptr)
    n = 1 << 26
    tab, idx, out = dp.alloc(0, 4 << 28), dp.alloc(0, 8 * n), dp.alloc(0, 4 * n)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(si.SEED0 + 2000)
    for lg in (16, 20, 22, 24, 26, 28):
        dp.view(idx, 8 * n).view(torch.int64).random_(0, 1 << lg, generator=gen)
        kargs = gd.gd_args_gather(out, tab, idx, n)
        row = {}
        for name, mode in both:
            sec = solo_avg_seconds(torch, st, lambda: gd.gd_launch_fenced(dp.pool, 0, gd.GD_K_GATHER32_I64, kargs, stream=st.cuda_stream, mode=mode), max(3, args.steps // 2))
            row[name + "_us"], row[name + "_Gloads_per_s"] = round(sec * 1e6, 1), round(n / sec / 1e9, 1)
        res["gather_i64_2^26_indices"][f"table_{4 << lg >> 20 if lg >= 18 else 0.25}_MiB"] = row
        log(f"[shapes] gather, table of 2^{lg} elements: fenced {row['fenced_us']} / unfenced {row['unfenced_us']} us ({row['fenced_Gloads_per_s']} G loads/s)")
    dp.close()
    return res


# ---------------------------------------------------------------------------------
# the paper's three bounds-checking rules side by side; cache-resident regime; host path
# ---------------------------------------------------------------------------------

def run_modes(torch, gd, si, args):
    """Section 4.4 / 7.2 ordering (native < bitwise < modulo < checking) and the
    Section 7.4 question (what the fence costs when data sit in cache), on one
    tenant with a 4 GiB partition; Section 7.6's host-side costs per call."""
    log("[modes] none / bitwise / modulo / checking / hardware checking on one tenant")
    dp = DevPool(torch, gd, [2 * GiB])                 # below 4 GiB: the hardware-checked rule addresses it with 32 bits
    counters = torch.zeros(4, dtype=torch.int64, device="cuda")
    gd.gd_pool_set_fault_counters(dp.pool, counters.data_ptr(), 4)
    st = torch.cuda.Stream()
    g = si.rng(6, 0)
    modes = (("none", gd.GD_FENCE_NONE), ("bitwise", gd.GD_FENCE_BITWISE), ("modulo", gd.GD_FENCE_MODULO), ("check", gd.GD_FENCE_CHECK),
             ("hwcheck", gd.GD_FENCE_HWCHECK))
    res = {"workload": "1 tenant, 2 GiB partition, all accesses in bounds: fp32 triad 2^26 (HBM resident); triad repeated inside one launch over working sets resident in L1, L2 and the Infinity Cache (each workgroup re-reads its own 3 KiB); gather 2^24 with int64 indices"}

    def sweep(label, kid, kargs, work, reps, unit="GBps", scale=1e9):
        out = {}
        for name, mode in modes:
            sec = solo_avg_seconds(torch, st, lambda: gd.gd_launch_fenced(dp.pool, 0, kid, kargs, stream=st.cuda_stream, mode=mode), reps)
            out[name + "_" + unit] = work / sec / scale
            out[name + "_us"] = sec * 1e6
        for name, _ in modes[1:]:
            out[name + "_overhead_pct"] = pct_overhead(out[name + "_" + unit], out["none_" + unit])
        log(f"[modes] {label}: " + ", ".join(f"{n} {out[n + '_us']:.2f} us" for n, _ in modes)
            + " | overhead " + ", ".join(f"{n} {out[n + '_overhead_pct']:+.1f} %" for n, _ in modes[1:]))
        res[label] = out

    n = 1 << 26
    a, b, c = (dp.alloc(0, 4 * n) for _ in range(3))
    host = np.empty(n, np.float32)
    for ptr, part in ((b, 1), (c, 2)):
        si.fill_chunked(host, 6, part, "uniform", threads=16)
        dp.upload(0, ptr, host)
    sweep("triad_hbm_2^26", gd.GD_K_TRIAD, gd.gd_args_triad(a, b, c, n, 0.5, 0), 12 * n, args.steps)
    # Section 7.4 / Fig. 5: what the fence costs when the data sit in a cache.  The triad's repeat field re-runs
    # the pass inside one launch (no nontemporal hint then); every workgroup re-reads its own 3 KiB, so the grid
    # decides which cache holds the working set.
    #   L1: 2048 single-wavefront workgroups, 8 per compute unit = 24 KiB per 32 KiB vector cache
    #   L2: 24 MiB over 8 XCDs = 3 MiB per 4 MiB L2, 32 workgroups (96 KiB) per compute unit, so L1 misses
    #   Infinity Cache: 48 MiB
    regimes = (("triad_L1_resident_2^19_x4000", 1 << 19, 4000, 0), ("triad_L2_resident_2^21_x1000", 1 << 21, 1000, 0),
               ("triad_infinity_cache_resident_2^22_x200", 1 << 22, 200, 0),
               # the same L1 regime through pointers that are not 16-byte aligned: 4-byte accesses, each fenced per lane
               # -- the per-access cost the paper's 8-cycles-against-28 model is about
               ("triad_L1_resident_per_lane_fence_2^19_x1000", 1 << 19, 1000, 4))
    for label, small, repeat, shift in regimes:
        sweep(label, gd.GD_K_TRIAD, gd.gd_args_triad(a + shift, b + shift, c + shift, small, 0.5, repeat), 12 * small * repeat,
              max(3, args.steps // 4))
    ng = 1 << 24
    idx = dp.alloc(0, 8 * ng)
    dp.upload(0, idx, g.integers(0, n, size=ng, dtype=np.int64))
    sweep("gather_i64_2^24", gd.GD_K_GATHER32_I64, gd.gd_args_gather(a, b, idx, ng), 16 * ng, args.steps)
    # the reduction, the normalisation and the GEMM under the five rules (configuration 5 / 4 shapes)
    ns = 1 << 27
    ws, sout = dp.alloc(0, gd.GD_SUM_WORKSPACE), dp.alloc(0, 256)
    sweep("sum_2^27", gd.GD_K_SUM_F32, gd.gd_args_sum(sout, b, ws, ns), 4 * ns, args.steps)        # b and c are adjacent: 2^27 values from b on
    rows, cols = 4096, 8192
    x, y, gain = dp.alloc(0, 2 * rows * cols), dp.alloc(0, 2 * rows * cols), dp.alloc(0, 2 * cols)
    dp.view(x, 2 * rows * cols).view(torch.bfloat16).normal_()
    dp.view(gain, 2 * cols).view(torch.bfloat16).uniform_(0.5, 1.5)
    sweep("rmsnorm_4096x8192", gd.GD_K_RMSNORM_BF16, gd.gd_args_rmsnorm(y, x, gain, rows, cols, 1e-6, 0), 4 * rows * cols, args.steps)
    M = 8192
    A, B, Cc = (dp.alloc(0, 2 * M * M) for _ in range(3))
    dp.view(A, 2 * M * M).view(torch.bfloat16).normal_(0.0, M ** -0.5)
    dp.view(B, 2 * M * M).view(torch.bfloat16).normal_()
    # every rule runs the DMA-ring kernel here (modulo and checking with A, B and C fenced once each, hardware
    # checking with buffer loads to the LDS)
    sweep("gemm_8192^3_bf16", gd.GD_K_GEMM_BF16, gd.gd_args_gemm(Cc, A, B, M, M, M, 1), 2.0 * M ** 3, max(3, args.steps // 2), unit="TFLOPs", scale=1e12)
    # Section 4.4's latency model (Figure 5: cycles of the fence against cycles of an access that hits L1, L2 or
    # goes to memory): one thread follows a random cycle over the cache lines of a footprint, every load fenced
    # per lane and dependent on the one before.  The table overwrites a (and b, c for the largest footprint).
    clk, cout = dp.alloc(0, 256), dp.alloc(0, 256)
    lat = {}
    for label, footprint, steps, warm in (("L1_16KiB", 16 << 10, 100000, False), ("L2_1MiB", 1 << 20, 100000, False),
                                          ("infinity_cache_64MiB", 64 << 20, 50000, True), ("hbm_512MiB", 512 << 20, 20000, False)):
        tab_host, first = si.chase_table(g, footprint)
        dp.upload(0, a, tab_host)
        del tab_host
        if warm:        # one walk over the whole cycle brings every line into the Infinity Cache
            gd.gd_launch_fenced(dp.pool, 0, gd.GD_K_CHASE, gd.gd_args_chase(cout, clk, a, footprint // 128, first, 0, 1, 0), stream=st.cuda_stream)
        else:           # nothing of the table is left in a cache by the upload: 512 MiB of other traffic in between
            gd.gd_launch_fenced(dp.pool, 0, gd.GD_K_GEMM_BF16, gd.gd_args_gemm(Cc, A, B, M, M, M, 1), stream=st.cuda_stream)
            gd.gd_launch_fenced(dp.pool, 0, gd.GD_K_RMSNORM_BF16, gd.gd_args_rmsnorm(y, x, gain, rows, cols, 1e-6, 0), stream=st.cuda_stream)
        row = {}
        at = first
        for name, mode in modes:
            best = None
            for _ in range(3):
                # every walk goes on where the last one ended: in the large footprints it meets lines no cache holds yet
                gd.gd_launch_fenced(dp.pool, 0, gd.GD_K_CHASE, gd.gd_args_chase(cout, clk, a, steps, at, 0, 1, 0), stream=st.cuda_stream, mode=mode)
                torch.cuda.synchronize()
                at = int(dp.view(cout, 4).cpu().numpy().view(np.uint32)[0])
                cycles, ticks = (int(v) for v in dp.view(clk, 16).cpu().numpy().view(np.uint64))
                if best is None or cycles < best[0]:
                    best = (cycles, ticks)
            row[name] = {"cycles_per_access": best[0] / steps, "ns_per_access": best[1] * 10.0 / steps}
        for name, _ in modes[1:]:
            row[name]["fence_cycles"] = row[name]["cycles_per_access"] - row["none"]["cycles_per_access"]
        lat[label] = row
        log(f"[modes] dependent fenced load, {label}: " + ", ".join(f"{n} {row[n]['cycles_per_access']:.0f} cycles ({row[n]['ns_per_access']:.0f} ns)" for n, _ in modes))
    res["latency_of_a_fenced_access"] = lat
    res["check_faults_counted"] = int(counters.sum().item())       # all accesses were in bounds: must be 0

    # host path, per call, Python binding included (the trivial call shows the binding's own share)
    def per_call_ns(fn, reps=20000):
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        return (time.perf_counter() - t0) / reps * 1e9
    torch.cuda.synchronize()
    kargs = gd.gd_args_store_tid(a, 0, 1, 0)                        # n = 0: lookup + augmentation, no launch
    host_ns = {
        "binding_trivial_call": per_call_ns(lambda: gd.gd_kernel_count()),
        "gd_check_copy": per_call_ns(lambda: gd.gd_check_copy(dp.pool, 0, a, 4096)),
        "gd_alloc_plus_gd_free": per_call_ns(lambda: gd.gd_free(dp.pool, 0, gd.gd_alloc(dp.pool, 0, 4096))),
        "gd_launch_fenced_lookup_and_augmentation_only": per_call_ns(lambda: gd.gd_launch_fenced(dp.pool, 0, gd.GD_K_STORE_TID, kargs, stream=st.cuda_stream)),
    }
    kargs1 = gd.gd_args_store_tid(a, 64, 1, 0)
    host_ns["gd_launch_fenced_with_launch"] = per_call_ns(lambda: gd.gd_launch_fenced(dp.pool, 0, gd.GD_K_STORE_TID, kargs1, stream=st.cuda_stream), 5000)
    torch.cuda.synchronize()
    res["host_ns_per_call"] = {k: round(v, 1) for k, v in host_ns.items()}
    log("[modes] host ns per call: " + ", ".join(f"{k} {v:.0f}" for k, v in host_ns.items()))
    # The same path timed inside the library (no binding in the figures), against the bare HIP launch call of the
    # same kernel: Section 7.6's Table 5 (lookup and augmentation against the launch itself).
    native = {}
    for label, mode in (("bitwise", gd.GD_FENCE_BITWISE), ("modulo", gd.GD_FENCE_MODULO), ("unfenced", gd.GD_FENCE_NONE)):
        gd.gd_probe_host_path(dp.pool, 0, a, 2000, stream=st.cuda_stream, mode=mode)             # warm
        up_to, with_launch, bare = gd.gd_probe_host_path(dp.pool, 0, a, 20000, stream=st.cuda_stream, mode=mode)
        native[label] = {"lookup_and_augmentation_ns": round(up_to, 1), "gd_launch_fenced_ns": round(with_launch, 1),
                         "bare_hip_launch_ns": round(bare, 1), "library_share_of_launch_pct": round(100.0 * (with_launch - bare) / bare, 1)}
        log(f"[modes] host path inside the library, {label}: up to the launch {up_to:.0f} ns, with the launch {with_launch:.0f} ns, "
            f"bare HIP launch {bare:.0f} ns")
    res["host_ns_per_call_native"] = native
    dp.close()
    return res


# ---------------------------------------------------------------------------------
# CPU baseline: the oracle as it stands (its OpenMP build) on the host cores of this machine
# ---------------------------------------------------------------------------------

def cpu_baseline(si):
    """Times the oracle on bounded samples of every configuration's kernels.  `value` is the leg
    that corresponds to the headline (configuration 3: copy + triad); the others are under `legs`."""
    from oracle import kernels as ok
    L = ok.lib(openmp=True)
    cores = int(L.gdo_threads())
    log(f"[cpu] timing the oracle (plain C, OpenMP build, {cores} threads; os.cpu_count() = {os.cpu_count()})")
    legs = {}

    def timed(fn, repeats=3):
        """Best wall-clock of `repeats` runs (every leg leaves the same image each time)."""
        best = float("inf")
        for _ in range(repeats):
            t0 = time.perf_counter()
            fn()
            best = min(best, time.perf_counter() - t0)
        return best

    def run(sim, row, name, *a):
        sim.run(name, row, ok.MODE_BITWISE, *a, openmp=True)
        assert sim.last[0] == 0 and sim.last[1] == 0

    # configuration 3: one tenant's copy + triad at full size (1/8 of a round), seeded scalar
    n = 1 << 28
    base, size = 1 << 40, 16 * GiB
    sim = ok.SimPool(base, 3 * 4 * n, 0)
    a, b, c = base, base + 4 * n, base + 8 * n
    si.fill_chunked(sim.view(b, np.float32, n), 3, 101, "uniform", threads=8)
    si.fill_chunked(sim.view(c, np.float32, n), 3, 201, "uniform", threads=8)
    s_val = float(si.uniform_f32(si.rng(3, 0), 1)[0])
    sec = timed(lambda: (run(sim, (base, size), "copy", a, b, n), run(sim, (base, size), "triad", a, b, c, s_val, n)))
    legs["c3_copy_triad"] = {"value": (8 + 12) * n / sec / 1e9, "unit": "GB/s", "seconds": sec,
                             "sample": "fenced copy + triad of one tenant, 2^28 fp32 elements per array: 1/8 of a round"}
    # configuration 5: the sum on the same array
    sec = timed(lambda: run(sim, (base, size), "sum_f32", a, b, 1 << 27))
    legs["c5_sum"] = {"value": 4 * (1 << 27) / sec / 1e9, "unit": "GB/s", "seconds": sec, "sample": "fp32 sum of 2^27 values (full size)"}
    del sim

    # configuration 2: gather then scatter over the full 2^26 table, first 2^25 of the 2^26 indices, in bounds
    tab_n, m = 1 << 26, 1 << 25
    base, size = 1 << 40, GiB
    sim = ok.SimPool(base, size, 0)
    tab, idx, out = base, base + 4 * tab_n, base + 4 * tab_n + 8 * tab_n
    si.fill_chunked(sim.view(tab, np.float32, tab_n), 2, 1, "normal", threads=8)
    sim.view(idx, np.int64, m)[:] = si.rng(2, 0).integers(0, tab_n, size=m, dtype=np.int64)
    sec_g = timed(lambda: run(sim, (base, size), "gather32_i64", out, tab, idx, m))
    sec_s = timed(lambda: run(sim, (base, size), "scatter_f32_i64", tab, out, idx, -1.0, m))
    legs["c2_gather"] = {"value": 16 * m / sec_g / 1e9, "unit": "GB/s", "seconds": sec_g, "sample": "table 2^26, the first 2^25 of 2^26 int64 indices (in bounds)"}
    legs["c2_scatter"] = {"value": 16 * m / sec_s / 1e9, "unit": "GB/s", "seconds": sec_s, "sample": "same indices, scatter back into the table"}
    # configuration 5: int32 gather (2^24 indices, full size) on the same table
    ng = 1 << 24
    sim.view(idx, np.int32, ng)[:] = si.rng(5, 1).integers(0, ng, size=ng, dtype=np.int64).astype(np.int32)
    sec = timed(lambda: run(sim, (base, size), "gather32_i32", out, tab, idx, ng))
    legs["c5_gather_i32"] = {"value": 12 * ng / sec / 1e9, "unit": "GB/s", "seconds": sec, "sample": "2^24 int32 indices over a 2^24 table (full size, in bounds)"}
    # configuration 5: RMSNorm 4096 x 8192 (full size)
    rows, cols = 4096, 8192
    x, y, gain = base, base + 2 * rows * cols, base + 4 * rows * cols
    g5 = si.rng(5, 2)
    sim.view(x, np.uint16, rows * cols)[:] = si.f32_to_bf16_bits(si.normal_f32(g5, rows * cols))
    sim.view(gain, np.uint16, cols)[:] = si.f32_to_bf16_bits(si.uniform_f32(g5, cols, 0.5, 1.5))
    sec = timed(lambda: run(sim, (base, size), "rmsnorm_bf16", y, x, gain, rows, cols, 1e-6))
    legs["c5_rmsnorm"] = {"value": 4 * rows * cols / sec / 1e9, "unit": "GB/s", "seconds": sec, "sample": "bf16 4096 x 8192 (full size)"}
    # configuration 4: a slab of rows of the 8192^3 product with the oracle's triple loop, scaled up; and the
    # whole product with NumPy's fp64 matmul (a library routine, labelled as such)
    M = N = K = 8192
    slab = 256
    A, B, Cc = base, base + 2 * M * K, base + 4 * M * K
    g4 = si.rng(4, 3)
    sim.view(A, np.uint16, slab * K)[:] = si.f32_to_bf16_bits(si.normal_f32(g4, slab * K) * np.float32(K ** -0.5))
    sim.view(B, np.uint16, N * K)[:] = si.f32_to_bf16_bits(si.normal_f32(g4, N * K))
    sec = timed(lambda: run(sim, (base, size), "gemm_bf16", Cc, A, B, M, N, K, 1, 0, slab, 0, N), repeats=1)   # the long leg: once
    legs["c4_gemm_oracle"] = {"value": 2.0 * slab * N * K / sec / 1e12, "unit": "TFLOP/s", "seconds": sec, "kind": "extrapolated",
                              "sample": f"rows 0..{slab} of C (1/{M // slab} of the product); the whole product would take {sec * M / slab:.0f} s"}
    Bf = si.bf16_bits_to_f32(sim.view(B, np.uint16, N * K)).reshape(N, K).astype(np.float64)
    Af = np.ascontiguousarray(np.tile(si.bf16_bits_to_f32(sim.view(A, np.uint16, slab * K)).reshape(slab, K), (2048 // slab, 1)).astype(np.float64))
    sec = timed(lambda: Af @ Bf.T)
    legs["c4_gemm_numpy_fp64"] = {"value": 2.0 * Af.shape[0] * N * K / sec / 1e12, "unit": "TFLOP/s", "seconds": sec, "kind": "library-backed",
                                  "sample": "NumPy fp64 matmul of a 2048 x 8192 by 8192 x 8192 product (1/4 of the rows)"}
    del sim, Af, Bf
    for k, v in legs.items():
        v["value"] = round(v["value"], 4)
        v["seconds"] = round(v["seconds"], 3)
        log(f"[cpu] {k}: {v['value']} {v['unit']} ({v['seconds']} s)")
    head = legs["c3_copy_triad"]
    return {"value": head["value"], "unit": "GB/s", "cores": cores, "kind": "oracle", "sample": head["sample"],
            "seconds": head["seconds"], "timing": "best of 3 runs per leg", "host_cpu_count": os.cpu_count(), "legs": legs}


def read_traffic():
    """HBM bytes per fenced triad launch from the committed rocprofv3 --pmc summary, if any."""
    path = os.path.join(ROOT, "profiles", "pmc_fence_overhead_and_traffic.md")
    try:
        for ln in open(path):
            if ln.startswith("traffic_bytes_per_launch:"):
                return float(ln.split(":")[1])
    except OSError:
        pass
    return None


def main():
    global PREWARM_MS
    args = parse()
    PREWARM_MS = args.prewarm_ms
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (tenants are streams of one context); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2401_09290_amd as gd
    import synth_inputs as si
    gd.lib()   # fails loudly if the HIP library has not been built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    runners = {"c1": run_c1, "c2": run_c2, "c3": run_c3, "c4": run_c4, "c5": run_c5, "modes": run_modes, "power": run_power, "gatherpolicy": run_gatherpolicy, "shapes": run_shapes}
    wanted = [c.strip() for c in args.configs.split(",") if c.strip()]
    per = {}
    for c in wanted:
        t0 = time.perf_counter()
        per[c] = runners[c](torch, gd, si, args)
        per[c]["bench_seconds"] = round(time.perf_counter() - t0, 1)
    out = {
        "metric": "fenced HBM GB/s, 8 tenants on 8 streams (copy + triad); GEMM TFLOP/s and % overhead vs unfenced under per_config",
        "value": None, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": None, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "configs[2]: 8 tenants x 16 GiB power-of-two partitions on 8 concurrent HIP streams, fenced STREAM copy + triad, fp32, 2^28 elements per array, all accesses in bounds"},
        "per_config": per,
    }
    if "c3" in per:
        c3 = per["c3"]
        out["value"] = round(c3["fenced_GBps"], 1)
        out["ms_per_step"] = round(c3["ms_per_round_fenced"], 4)
        tri = c3["solo"]["triad_fenced"]
        out["roofline"] = {"bound": "hbm", "kernel": "k_stream<V_BIT64, triad, nontemporal>", "achieved": round(tri["GBps"], 1),
                           "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(tri["GBps"] / HBM_PEAK_GBPS, 4),
                           "avg_launch_ms": round(tri["avg_launch_ms"], 4), "bytes_per_launch": c3["triad_bytes_per_launch"],
                           "traffic": read_traffic()}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(si)
    print(json.dumps(out), flush=True)
    log(f"[bench] done at {time.time():.3f}")


if __name__ == "__main__":
    main()
