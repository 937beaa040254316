"""Summarise a rocprofv3 kernel trace (``--kernel-trace --output-format csv``).

Tenants run on concurrent streams, so the begin-to-end time of a dispatch that
shares the GPU with other dispatches says little about the kernel itself.  This
tool prints, per kernel, the usual statistics over all dispatches and the same
statistics over the dispatches that ran ALONE (their interval overlaps no other
dispatch of the trace) -- the figure to hold against a per-launch roofline.

usage: python -m paper_2401_09290_amd.rocprof_summary <kernel_trace.csv> [name-filter]
"""
import csv
import sys


def load(path):
    rows = []
    with open(path, newline="") as f:
        for r in csv.DictReader(f):
            rows.append((r["Kernel_Name"], int(r["Start_Timestamp"]), int(r["End_Timestamp"]),
                         r.get("VGPR_Count", ""), r.get("Accum_VGPR_Count", ""), r.get("SGPR_Count", ""),
                         r.get("Scratch_Size", ""), r.get("LDS_Block_Size", "")))
    return rows


def alone_flags(rows):
    """True for dispatches whose [start, end) overlaps no other dispatch."""
    order = sorted(range(len(rows)), key=lambda i: rows[i][1])
    alone = [True] * len(rows)
    latest_end, latest_i = -1, -1
    for i in order:
        start, end = rows[i][1], rows[i][2]
        if start < latest_end:
            alone[i] = False
            alone[latest_i] = False
        if end > latest_end:
            latest_end, latest_i = end, i
    return alone


def short(name):
    name = name.replace("void ", "")
    cut = name.find("(")
    return name[:cut] if cut > 0 else name


def summarise(path, needle=""):
    rows = load(path)
    alone = alone_flags(rows)
    stats = {}
    for r, a in zip(rows, alone):
        if needle and needle not in r[0]:
            continue
        s = stats.setdefault(short(r[0]), {"all": [], "alone": [], "regs": r[3:8]})
        d = r[2] - r[1]
        s["all"].append(d)
        if a:
            s["alone"].append(d)
    lines = ["kernel | calls | avg us (all) | calls alone | avg us (alone) | min us | VGPR/AGPR/SGPR | scratch | LDS",
             "---|---|---|---|---|---|---|---|---"]
    for name, s in sorted(stats.items(), key=lambda kv: -sum(kv[1]["all"])):
        al = s["alone"]
        lines.append(f"{name} | {len(s['all'])} | {sum(s['all']) / len(s['all']) / 1e3:.1f} | {len(al)} | "
                     f"{(sum(al) / len(al) / 1e3) if al else float('nan'):.1f} | {min(s['all']) / 1e3:.1f} | "
                     f"{s['regs'][0]}/{s['regs'][1]}/{s['regs'][2]} | {s['regs'][3]} | {s['regs'][4]}")
    return "\n".join(lines)


if __name__ == "__main__":
    if len(sys.argv) < 2:
        sys.exit(__doc__)
    print(summarise(sys.argv[1], sys.argv[2] if len(sys.argv) > 2 else ""))
