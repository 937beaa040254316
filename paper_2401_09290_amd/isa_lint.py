"""Coverage audit of the fenced kernels on the gfx950 ISA the compiler emits.

The paper's patcher guarantees by construction that every load and store of a
sandboxed kernel is preceded by the fence (Section 4.3) and reports how many
loads and stores it instrumented per library (Table 3) and how many extra
registers the fence costs (Section 7.3).  Here the kernels are written fenced, so
the same guarantee is checked after the fact, on the assembly text produced by
``hipcc -S`` for each source file:

* no kernel uses flat_* accesses, indirect branches (s_setpc / s_swappc) or --
  outside the GEMM, which may spill a few registers to scratch -- scratch memory;
* in every kernel built with the 32-bit fence (variant 1) each global_load,
  global_store, global_atomic and global_load_lds addresses memory as
  "SGPR base + 32-bit VGPR offset", and the instruction that last wrote that
  offset register is the fence's ``v_and_b32`` with an SGPR mask;
* in every kernel built with the 64-bit fence (variant 2) each global access
  uses a 64-bit VGPR address whose high word was last written by ``v_or_b32``
  with an SGPR operand (the OR with the partition base, after the AND);
* per kernel: loads, stores, fence instructions, VGPR/SGPR counts and the
  register delta against the unfenced build of the same kernel.

usage: python -m paper_2401_09290_amd.isa_lint            (prints the table, exit 1 on a violation)
"""
import os
import re
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
HIP_SOURCES = ["kernels_stream.hip", "kernels_indexed.hip", "kernels_reduce.hip", "gemm.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-S", "--cuda-device-only", "-Wno-unused-command-line-argument"]

MEM_RE = re.compile(r"^\s*(global_load_lds_\w+|global_load_\w+|global_store_\w+|global_atomic_\w+)\s+(.*)$")
# the counters the checking variant bumps live in manager-owned memory and are not fenced by design
UNFENCED_OK = ("global_atomic_add_x2",)


def demangle(names):
    """Readable kernel names via c++filt if it is there; otherwise a minimal reading of
    the Itanium names this library produces (namespace gd, integer template arguments)."""
    try:
        out = subprocess.run(["c++filt"] + names, capture_output=True, text=True)
        if out.returncode == 0 and len(out.stdout.splitlines()) == len(names):
            return out.stdout.splitlines()
    except OSError:
        pass
    pretty = []
    for n in names:
        m = re.match(r"^_ZN2gd\d+([a-z_0-9]+?)I(.*?)EEv", n)
        if not m:
            pretty.append(n)
            continue
        args = re.findall(r"L[ib](\d+)E", m.group(2))
        pretty.append(f"void gd::{m.group(1)}<{', '.join(args)}>(")
    return pretty


def kernels_of(asm_text):
    """name -> list of instruction lines, plus metadata dicts, from one .s file."""
    bodies, meta = {}, {}
    cur = None
    for ln in asm_text.splitlines():
        m = re.match(r"^(_Z\w+):\s", ln)
        if m:
            cur = m.group(1)
            bodies[cur] = []
            continue
        if cur and re.match(r"^\s*s_endpgm", ln):
            bodies[cur].append(ln)
            cur = None
            continue
        if cur is not None:
            code = ln.split(";")[0].rstrip()
            if code.strip() and not code.strip().startswith("."):
                bodies[cur].append(code)
    # metadata block: .amdhsa_kernel NAME ... .amdhsa_next_free_vgpr N
    for m in re.finditer(r"\.amdhsa_kernel (\S+)(.*?)\.end_amdhsa_kernel", asm_text, re.S):
        name, blk = m.group(1), m.group(2)
        def grab(key):
            g = re.search(r"\." + key + r"\s+(\d+)", blk)
            return int(g.group(1)) if g else -1
        meta[name] = {"vgpr": grab("amdhsa_next_free_vgpr"), "sgpr": grab("amdhsa_next_free_sgpr"),
                      "scratch": grab("amdhsa_private_segment_fixed_size"), "accum": grab("amdhsa_accum_offset")}
    return bodies, meta


def writes_reg(line, reg):
    """Does this instruction write VGPR number `reg` (as its first operand)?"""
    m = re.match(r"^\s*(\w+)\s+([^,\s]+)", line)
    if not m or m.group(1).startswith(("s_", "global_store", "ds_write", "buffer_store", "global_load_lds")):
        return False
    dst = m.group(2)
    r = re.match(r"^v(\d+)$", dst)
    if r:
        return int(r.group(1)) == reg
    r = re.match(r"^v\[(\d+):(\d+)\]$", dst)
    return bool(r) and int(r.group(1)) <= reg <= int(r.group(2))


def last_writer(body, idx, reg):
    order = list(range(idx - 1, -1, -1)) + list(range(len(body) - 1, idx, -1))   # backwards, wrapping (loops)
    for j in order:
        if writes_reg(body[j], reg):
            return body[j].strip()
    return None


def last_scalar_writer(body, idx, sreg):
    for j in range(idx - 1, -1, -1):
        m = re.match(r"^\s*(s_\w+)\s+([^,\s]+)", body[j])
        if not m or m.group(1).startswith(("s_cmp", "s_cbranch", "s_waitcnt", "s_barrier", "s_nop", "s_branch")):
            continue
        dst = m.group(2)
        r = re.match(r"^s(\d+)$", dst)
        if r and int(r.group(1)) == sreg:
            return body[j].strip()
        r = re.match(r"^s\[(\d+):(\d+)\]$", dst)
        if r and int(r.group(1)) <= sreg <= int(r.group(2)):
            return body[j].strip()
    return None


def lint_kernel(name, pretty, body, variant):
    problems, loads, stores, fences = [], 0, 0, 0
    for i, ln in enumerate(body):
        op = ln.strip().split()[0] if ln.strip() else ""
        if op.startswith("flat_"):
            problems.append(f"{pretty}: flat access: {ln.strip()}")
        if op in ("s_setpc_b64", "s_swappc_b64"):
            problems.append(f"{pretty}: indirect branch: {ln.strip()}")
        if op.startswith("v_and_b32") and re.search(r"\bs\d+\b", ln):
            fences += 1
        m = MEM_RE.match(ln)
        if not m:
            continue
        inst, ops = m.group(1), [o.strip() for o in m.group(2).split(",")]
        is_store = inst.startswith("global_store")
        loads += (not is_store) and not inst.startswith("global_atomic")
        stores += is_store
        if inst in UNFENCED_OK or variant not in (1, 2):
            continue
        if inst.startswith("global_load_lds"):
            addr, base = ops[0], ops[1] if len(ops) > 1 else ""
        elif is_store:
            addr, base = ops[0], ops[2] if len(ops) > 2 else ""
        else:
            addr, base = ops[1], ops[2] if len(ops) > 2 else ""
        base = base.split()[0] if base else ""
        if variant == 1:
            r = re.match(r"^v(\d+)$", addr)
            if not r or not base.startswith("s["):
                problems.append(f"{pretty}: 32-bit fence but not SGPR-base + VGPR-offset: {ln.strip()}")
                continue
            w = last_writer(body, i, int(r.group(1)))
            if not (w and w.startswith("v_and_b32") and re.search(r"\bs\d+\b", w)):
                problems.append(f"{pretty}: offset v{r.group(1)} of `{ln.strip()}` last written by `{w}`")
        else:
            r = re.match(r"^v\[(\d+):(\d+)\]$", addr)
            sb = re.match(r"^s\[(\d+):(\d+)\]$", base)
            if sb and re.match(r"^v\d+$", addr):
                # a wave-uniform address fenced on the scalar unit: s_or_b64 into the base pair, zero offset
                sw = last_scalar_writer(body, i, int(sb.group(2)))
                vw = last_writer(body, i, int(addr[1:]))
                if not (sw and sw.startswith("s_or_b") and vw and re.match(r"^v_mov_b32\w*\s+v\d+,\s*0$", vw)):
                    problems.append(f"{pretty}: scalar address of `{ln.strip()}` last written by `{sw}` / offset by `{vw}`")
                continue
            if not r or base != "off":
                problems.append(f"{pretty}: 64-bit fence but not a 64-bit VGPR address: {ln.strip()}")
                continue
            w = last_writer(body, i, int(r.group(2)))
            if not (w and w.startswith("v_or_b32") and re.search(r"\bs\d+\b", w)):
                problems.append(f"{pretty}: high word v{r.group(2)} of `{ln.strip()}` last written by `{w}`")
    return problems, loads, stores, fences


def run(verbose=True):
    rows, problems = [], []
    with tempfile.TemporaryDirectory() as tmp:
        for src in HIP_SOURCES:
            out = os.path.join(tmp, src + ".s")
            res = subprocess.run(["hipcc", *FLAGS, "-o", out, os.path.join(CSRC, src)], capture_output=True, text=True)
            if res.returncode != 0:
                raise RuntimeError(res.stderr)
            bodies, meta = kernels_of(open(out).read())
            names = [n for n in bodies if "gd" in n]
            pretty = dict(zip(names, demangle(names)))
            for n in names:
                p = pretty[n].replace("void gd::", "").split("(")[0]
                v = re.search(r"<(\d)", p)
                variant = int(v.group(1)) if v else -1
                pr, ld, st, fc = lint_kernel(n, p, bodies[n], variant)
                md = meta.get(n, {})
                if md.get("scratch", 0) > 0 and "gemm" not in p:
                    pr.append(f"{p}: uses {md['scratch']} bytes of scratch")
                problems += pr
                rows.append((p, variant, ld, st, fc, md.get("vgpr", -1), md.get("sgpr", -1), md.get("scratch", -1)))
    base = {re.sub(r"<\d", "<0", r[0]): r for r in rows if r[1] == 0}
    lines = ["kernel | variant | loads | stores | fence v_and_b32 | VGPRs | SGPRs | scratch | VGPR delta vs unfenced | SGPR delta",
             "---|---|---|---|---|---|---|---|---|---"]
    for r in sorted(rows):
        b = base.get(re.sub(r"<\d", "<0", r[0]))
        dv = r[5] - b[5] if b else ""
        ds = r[6] - b[6] if b else ""
        lines.append(f"{r[0]} | {r[1]} | {r[2]} | {r[3]} | {r[4]} | {r[5]} | {r[6]} | {r[7]} | {dv} | {ds}")
    text = "\n".join(lines)
    if verbose:
        print(text)
        print(f"\n{len(rows)} kernels, {len(problems)} problem(s)")
        for p in problems:
            print("PROBLEM:", p)
    return rows, problems, text


if __name__ == "__main__":
    _, probs, _ = run()
    sys.exit(1 if probs else 0)
