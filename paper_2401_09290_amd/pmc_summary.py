"""Summarise rocprofv3 ``--pmc`` runs of ``bench.py`` into the tables kept under ``profiles/``.

Input: a directory with one sub-directory per counter run, each holding the
``*_counter_collection.csv`` that ``rocprofv3 --pmc ... --output-format csv`` writes:

    insts/   SQ_INSTS_VALU SQ_INSTS_SALU SQ_INSTS_VMEM SQ_INSTS_LDS SQ_WAVES
             SQ_INSTS_VALU_MFMA_BF16 SQ_VALU_MFMA_BUSY_CYCLES GRBM_GUI_ACTIVE
    fetch/   FETCH_SIZE          (KiB per dispatch, before calibration)
    write/   WRITE_SIZE

Counters are averaged per kernel over its dispatches.  The tables:

* instructions per dispatch and per wavefront, and the fence's cost in vector
  instructions per wavefront (each fenced kernel ``name<V, ...>`` against the unfenced
  build ``name<0, ...>`` of the same kernel);
* matrix-pipe utilisation of every kernel that issues MFMA instructions;
* bytes past the L2 per dispatch, FETCH_SIZE and WRITE_SIZE each scaled by what the
  same counter reads for the unfenced copy kernel, whose traffic is known
  (``--copy-elems`` 4-byte elements read and written once), against the algorithmic
  bytes of bench.py's default sizes.  The line ``traffic_bytes_per_launch:`` (the fenced
  triad of the headline configuration) is what bench.py reports as ``roofline.traffic``.

usage: python -m paper_2401_09290_amd.pmc_summary DIR [--copy-elems N]
"""
import argparse
import collections
import csv
import glob
import os
import re

XCDS = 8
SIMDS = 1024                      # 256 compute units x 4
VARIANTS = {0: "unfenced", 1: "bitwise, 32-bit offset", 2: "bitwise, 64-bit", 3: "modulo", 4: "checking",
            5: "hardware checking (buffer)"}

# algorithmic bytes per dispatch at bench.py's default sizes, by kernel (template arguments after the variant)
GiB, MiB = 1 << 30, 1 << 20
ALGORITHMIC = {
    "k_stream<V, 0, true>": 2 * GiB, "k_stream<V, 1, true>": 3 * GiB,
    "k_gather32<V, 1>": 16 << 26, "k_scatter_f32_i64<V>": 16 << 26, "k_gather32<V, 0>": 12 << 24,
    "k_sum_partial<V, false>": 4 << 27, "k_rmsnorm_bf16<V, 2, true>": 4 * 4096 * 8192, "k_gemm_ring<V>": 3 * 128 * MiB, "k_gemm_ring<V, false>": 3 * 128 * MiB, "k_gemm_ring<V, true>": 3 * 128 * MiB,
}


def short_name(kernel_name):
    name = kernel_name.split("(")[0].replace("void ", "").replace("gd::", "")
    return name.strip()


def variant_of(name):
    m = re.search(r"<(\d+)", name)
    return int(m.group(1)) if m else None


def generic(name):
    """k_stream<2, 1, true> -> k_stream<V, 1, true> (the key under which builds of one kernel are paired)."""
    return re.sub(r"<\d+", "<V", name, count=1)


def load(run_dir, needle="gd::"):
    """{kernel: {counter: mean over dispatches, 'dur_ns': mean, 'calls': n}} of one counter run."""
    files = sorted(glob.glob(os.path.join(run_dir, "**", "*counter_collection.csv"), recursive=True))
    if not files:
        return {}
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    for path in files:
        with open(path, newline="") as f:
            for r in csv.DictReader(f):
                if needle not in r["Kernel_Name"]:
                    continue
                k = short_name(r["Kernel_Name"])
                acc[k][r["Counter_Name"]].append(float(r["Counter_Value"]))
                acc[k]["dur_ns"].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    out = {}
    for k, counters in acc.items():
        out[k] = {c: sum(v) / len(v) for c, v in counters.items()}
        out[k]["calls"] = max(len(v) for c, v in counters.items() if c != "dur_ns")
    return out


def instruction_table(ins):
    lines = ["kernel | rule | waves | VALU | of which MFMA | SALU | VMEM | LDS | VALU per wave | SALU per wave",
             "---|---|---|---|---|---|---|---|---|---"]
    for k in sorted(ins):
        v = ins[k]
        w = v.get("SQ_WAVES") or 1.0
        lines.append(f"{k} | {VARIANTS.get(variant_of(k), '')} | {v.get('SQ_WAVES', 0):.0f} | {v.get('SQ_INSTS_VALU', 0):.0f} | "
                     f"{v.get('SQ_INSTS_VALU_MFMA_BF16', 0):.0f} | {v.get('SQ_INSTS_SALU', 0):.0f} | {v.get('SQ_INSTS_VMEM', 0):.0f} | "
                     f"{v.get('SQ_INSTS_LDS', 0):.0f} | {v.get('SQ_INSTS_VALU', 0) / w:.1f} | {v.get('SQ_INSTS_SALU', 0) / w:.1f}")
    return lines


def fence_cost(ins):
    """Per fenced kernel: vector and scalar instructions per wavefront minus those of the unfenced build."""
    base = {generic(k): v for k, v in ins.items() if variant_of(k) == 0}
    lines = ["kernel | rule | VALU per wave: fenced - unfenced | SALU per wave: fenced - unfenced | VALU overhead",
             "---|---|---|---|---"]
    rows = []
    for k in sorted(ins):
        b = base.get(generic(k))
        if variant_of(k) in (None, 0) or not b:
            continue
        v = ins[k]
        per = lambda d, c: d.get(c, 0) / (d.get("SQ_WAVES") or 1.0)
        dv, ds = per(v, "SQ_INSTS_VALU") - per(b, "SQ_INSTS_VALU"), per(v, "SQ_INSTS_SALU") - per(b, "SQ_INSTS_SALU")
        pct = 100.0 * dv / per(b, "SQ_INSTS_VALU") if per(b, "SQ_INSTS_VALU") else float("nan")
        rows.append((k, dv, ds, pct))
        lines.append(f"{k} | {VARIANTS.get(variant_of(k), '')} | {dv:+.1f} | {ds:+.1f} | {pct:+.1f} %")
    return lines, rows


def mfma_table(ins):
    lines = []
    for k in sorted(ins):
        v = ins[k]
        n = v.get("SQ_INSTS_VALU_MFMA_BF16", 0)
        if not n or "GRBM_GUI_ACTIVE" not in v:
            continue
        cycles = v["GRBM_GUI_ACTIVE"] / XCDS
        busy = v.get("SQ_VALU_MFMA_BUSY_CYCLES", 0)
        lines.append(f"* {k}: {n:.0f} MFMA instructions, SQ_VALU_MFMA_BUSY_CYCLES {busy:.0f} ({busy / n:.1f} per instruction) over "
                     f"{cycles:.0f} shader cycles x {SIMDS} SIMDs = {100.0 * busy / (cycles * SIMDS):.1f} % of the matrix-pipe cycles; "
                     f"shader clock during the kernel {cycles / v['dur_ns']:.2f} GHz (GRBM_GUI_ACTIVE / {XCDS} XCDs / duration; "
                     f"dispatches are serialised by the profiler, bench.py's timing is the reference for throughput)")
    return lines


def traffic_table(fetch, write, copy_elems):
    copy = [k for k in fetch if generic(k).startswith("k_stream<V, 0") and variant_of(k) == 0 and k in write]
    if not copy:
        return ["(no unfenced copy kernel in the counter runs: FETCH_SIZE / WRITE_SIZE cannot be calibrated)"], None
    ref = copy[0]
    known_kib = 4.0 * copy_elems / 1024.0
    cf, cw = known_kib / fetch[ref]["FETCH_SIZE"], known_kib / write[ref]["WRITE_SIZE"]
    lines = [f"Calibration on `{ref}` (reads and writes {4 * copy_elems} bytes once): FETCH_SIZE reads "
             f"{fetch[ref]['FETCH_SIZE']:.1f}, WRITE_SIZE reads {write[ref]['WRITE_SIZE']:.1f}; scale factors {cf:.5f} (fetch) and {cw:.5f} (write).",
             "",
             "kernel | rule | fetched bytes | written bytes | total | algorithmic | total / algorithmic",
             "---|---|---|---|---|---|---"]
    headline = None
    for k in sorted(set(fetch) & set(write)):
        fb = fetch[k]["FETCH_SIZE"] * cf * 1024.0
        wb = write[k]["WRITE_SIZE"] * cw * 1024.0
        alg = ALGORITHMIC.get(generic(k))
        ratio = f"{(fb + wb) / alg:.3f}" if alg else ""
        lines.append(f"{k} | {VARIANTS.get(variant_of(k), '')} | {fb:.4g} | {wb:.4g} | {fb + wb:.4g} | {alg or ''} | {ratio}")
        if generic(k) == "k_stream<V, 1, true>" and variant_of(k) == 2:
            headline = fb + wb
    return lines, headline


def summarise(root, copy_elems=1 << 28):
    ins, fetch, write = (load(os.path.join(root, d)) for d in ("insts", "fetch", "write"))
    out = ["## Instructions per dispatch", ""] + instruction_table(ins)
    cost, _ = fence_cost(ins)
    out += ["", "## Cost of the fence in instructions per wavefront", ""] + cost
    mf = mfma_table(ins)
    if mf:
        out += ["", "## Matrix-pipe utilisation", ""] + mf
    tr, headline = traffic_table(fetch, write, copy_elems)
    out += ["", "## Bytes past the L2 per dispatch", ""] + tr
    if headline is not None:
        out += ["", "Fenced triad of the headline configuration (`roofline.traffic` of bench.py):", "",
                f"traffic_bytes_per_launch: {headline:.0f}"]
    return "\n".join(out) + "\n"


if __name__ == "__main__":
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("root")
    ap.add_argument("--copy-elems", type=int, default=1 << 28)
    a = ap.parse_args()
    print(summarise(a.root, a.copy_elems), end="")
