"""Coverage audit of the fenced kernels on the gfx950 ISA the compiler emits.

The paper's patcher guarantees by construction that every load and store of a
sandboxed kernel is preceded by the fence (Section 4.3) and reports how many
loads and stores it instrumented per library (Table 3) and how many extra
registers the fence costs (Section 7.3).  Here the kernels are written fenced, so
the same guarantee is checked after the fact, on the assembly text produced by
``hipcc -S`` for each source file:

* no kernel uses flat_* accesses, indirect branches (s_setpc / s_swappc) or scratch
  memory;
* in every kernel built with the 32-bit fence (variant 1) each global_load,
  global_store, global_atomic and global_load_lds addresses memory as
  "SGPR base + 32-bit VGPR offset", and the instruction that last wrote that
  offset register is the fence's ``v_and_b32`` with an SGPR mask;
* in every kernel built with the 64-bit fence (variant 2) each global access
  uses a 64-bit VGPR address whose high word was last written by ``v_or_b32``
  with an SGPR operand (the OR with the partition base, after the AND);
* in both, an access through the scalar fence of a contiguous array uses as its base an
  SGPR pair that is the fence's ``s_or_b64`` result, or that result plus an offset
  (scalar add with carry), and as its offset a lane offset confined by an AND with a
  constant below 4096 (or zero);
* in every kernel built for the hardware-checked rule (variant 5) all accesses to tenant
  memory are buffer instructions with a VGPR offset and a zero SGPR offset (the range
  check covers exactly that offset), and there is no global_* access;
* the sum kernels that keep their partial sums in the library's own device array
  access that array unfenced (manager memory), and nothing else;
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
BUF_RE = re.compile(r"^\s*(buffer_load_\w+|buffer_store_\w+)\s+(.*)$")
LABEL_RE = re.compile(r"^(\.L\w+):$")
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
        if cur and re.match(r"^\.Lfunc_end\d+:", ln):        # a kernel may hold several s_endpgm: its text ends here
            cur = None
            continue
        if cur is not None:
            code = ln.split(";")[0].rstrip()
            if code.strip() and (not code.strip().startswith(".") or LABEL_RE.match(code.strip())):
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


NO_DEST = ("s_cmp", "s_cbranch", "s_branch", "s_waitcnt", "s_barrier", "s_nop", "s_endpgm", "s_setprio", "s_sleep",
           "s_bitcmp", "s_setreg", "s_sendmsg", "s_trap", "global_store", "ds_write", "buffer_store",
           "global_load_lds", "v_cmpx", "v_nop", "s_mov_b32 m0")
# instructions whose second operand is written as well (carry / scale outputs)
TWO_DEST = ("v_mad_u64_u32", "v_mad_i64_i32", "v_add_co_u32", "v_sub_co_u32", "v_subrev_co_u32", "v_addc_co_u32",
            "v_subb_co_u32", "v_subbrev_co_u32", "v_div_scale_f32", "v_div_scale_f64")


def _regs(operand):
    """('v'|'s', lo, hi) of a register operand, or None."""
    m = re.match(r"^([vs])(\d+)$", operand)
    if m:
        return m.group(1), int(m.group(2)), int(m.group(2))
    m = re.match(r"^([vs])\[(\d+):(\d+)\]$", operand)
    if m:
        return m.group(1), int(m.group(2)), int(m.group(3))
    return None


def dests(line):
    """Registers an instruction writes (explicit operands only; vcc, scc, exec and m0 are not tracked)."""
    code = line.strip()
    m = re.match(r"^(\w+)\s+(.*)$", code)
    if not m or LABEL_RE.match(code) or code.startswith(NO_DEST):
        return []
    op, ops = m.group(1), [o.strip().split()[0] for o in m.group(2).split(",") if o.strip()]
    out = []
    for k in range(2 if op.startswith(TWO_DEST) else 1):
        if k < len(ops) and _regs(ops[k]):
            out.append(_regs(ops[k]))
    return out


class Flow:
    """Control-flow graph of one kernel body and reaching definitions on it."""

    def __init__(self, body):
        self.body = body
        n = len(body)
        label_at = {}
        for i, ln in enumerate(body):
            m = LABEL_RE.match(ln.strip())
            if m:
                label_at[m.group(1)] = i
        self.preds = [[] for _ in range(n + 1)]            # instruction index -> indices it can be reached from
        for i, ln in enumerate(body):
            code = ln.strip()
            op = code.split()[0] if code else ""
            target = code.split()[-1] if op.startswith(("s_branch", "s_cbranch")) else None
            if target is not None and target in label_at:
                self.preds[label_at[target]].append(i)
            if not op.startswith(("s_branch", "s_endpgm")) and i + 1 < n:
                self.preds[i + 1].append(i)

    def reaching_at(self, idx, kind, reg):
        """Indices of the instructions whose write of `reg` can reach instruction idx; -1 stands for
        the value the register holds when the kernel starts."""
        found, seen, stack = set(), set(), list(self.preds[idx])
        if not stack:
            found.add(-1)
        while stack:
            j = stack.pop()
            if j in seen:
                continue
            seen.add(j)
            if any(k == kind and lo <= reg <= hi for (k, lo, hi) in dests(self.body[j])):
                found.add(j)
                continue
            if self.preds[j]:
                stack.extend(self.preds[j])
            else:
                found.add(-1)
        return found

    def reaching(self, idx, kind, reg):
        """The same as instruction texts ('ENTRY' for the kernel's start)."""
        return {"ENTRY" if j < 0 else self.body[j].strip() for j in self.reaching_at(idx, kind, reg)}


FENCE_AND32 = re.compile(r"^v_and_b32\w*\s+v\d+,\s*(s\d+,\s*v\d+|v\d+,\s*s\d+)$")
FENCE_OR32 = re.compile(r"^v_or_b32\w*\s+v\d+,\s*(s\d+,\s*v\d+|v\d+,\s*s\d+)$")
TILE_OR64 = re.compile(r"^s_or_b64\s+s\[\d+:\d+\],\s*s\[\d+:\d+\],\s*s\[\d+:\d+\]$")   # OR of two SGPR pairs (not vcc/exec)
LANE_CONFINED = re.compile(r"^v_and_b32\w*\s+v\d+,\s*(0x[0-9a-f]+|\d+),\s*v\d+$")
ZERO_V = re.compile(r"^v_mov_b32\w*\s+v\d+,\s*0$")
ZERO_S = re.compile(r"^s_mov_b(32|64)\s+s(\d+|\[\d+:\d+\]),\s*0$")


SCALAR_ADD = re.compile(r"^s_addc?_u32\s+s(\d+),\s*(s\d+|\S+),\s*(s\d+|\S+)$")


def fenced_scalar(flow, idx, sreg, depth=0, seen=None):
    """Is the SGPR `sreg`, as read by instruction idx, a fenced address word?  Every definition that
    reaches the read must be the fence's s_or_b64, the zero a never-taken path initialises it with, or a
    scalar add one of whose operands is such a word (fenced start + offset: the carry chain of a 64-bit
    add).  Returns (ok, saw_fence)."""
    seen = set() if seen is None else seen
    ok, saw = True, False
    for j in flow.reaching_at(idx, "s", sreg):
        if j < 0:
            return False, saw
        text = flow.body[j].strip()
        if TILE_OR64.match(text):
            saw = True
        elif ZERO_S.match(text):
            pass
        elif SCALAR_ADD.match(text) and depth < 6:
            if (j, sreg) in seen:
                saw = True                                # a loop-carried add: judged where the chain was entered
                continue
            seen.add((j, sreg))
            srcs = [o for o in SCALAR_ADD.match(text).groups()[1:] if re.match(r"^s\d+$", o)]
            sub = [fenced_scalar(flow, j, int(o[1:]), depth + 1, seen) for o in srcs]
            if not any(k and f for k, f in sub):
                return False, saw
            saw = True
        else:
            return False, saw
    return ok, saw


def lint_kernel(name, pretty, body, variant):
    problems, loads, stores, fences = [], 0, 0, 0
    tiles = own_ws_seen = 0
    own_ws = bool(re.search(r"k_sum_\w+<\d, (true|1)>", pretty))
    flow = Flow(body)
    for i, ln in enumerate(body):
        op = ln.strip().split()[0] if ln.strip() else ""
        if op.startswith("flat_"):
            problems.append(f"{pretty}: flat access: {ln.strip()}")
        if op in ("s_setpc_b64", "s_swappc_b64"):
            problems.append(f"{pretty}: indirect branch: {ln.strip()}")
        if FENCE_AND32.match(ln.strip()) or TILE_OR64.match(ln.strip()):
            fences += 1
        if variant == 5 and BUF_RE.match(ln):
            is_st = "store" in ln.split()[0]
            loads += not is_st
            stores += is_st
            fences += 1                                   # the descriptor's range check is the fence
            if not re.search(r"\boffen\b", ln) or re.search(r",\s*s\d+\s+offen", ln):
                problems.append(f"{pretty}: buffer access without a VGPR offset or with an SGPR offset: {ln.strip()}")
            continue
        m = MEM_RE.match(ln)
        if not m:
            continue
        inst, ops = m.group(1), [o.strip() for o in m.group(2).split(",")]
        is_store = inst.startswith("global_store")
        loads += (not is_store) and not inst.startswith("global_atomic")
        stores += is_store
        if variant == 5 and inst not in UNFENCED_OK and not own_ws:
            problems.append(f"{pretty}: hardware-checked rule but a global access: {ln.strip()}")
        if inst in UNFENCED_OK or variant not in (1, 2):
            continue
        if own_ws and ((is_store and "k_sum_partial" in pretty) or (not is_store and "k_sum_final" in pretty)):
            own_ws_seen += 1          # the library's own partial-sum array: manager memory, unfenced by design
            continue
        if inst.startswith("global_load_lds"):
            addr, base = ops[0], ops[1] if len(ops) > 1 else ""
        elif is_store:
            addr, base = ops[0], ops[2] if len(ops) > 2 else ""
        else:
            addr, base = ops[1], ops[2] if len(ops) > 2 else ""
        base = base.split()[0] if base else ""
        what = ln.strip()
        sb, va = _regs(base), _regs(addr)
        # Scalar tile fence (both bitwise variants): every definition of the base pair that
        # reaches the access is the fence's s_or_b64 (after its s_and_b64) -- or the zero a
        # never-taken path initialises it with -- and the offset is a lane offset confined
        # below the tile size by an AND with a constant, or zero.
        if sb and sb[0] == "s" and va and va[0] == "v" and va[1] == va[2]:
            bdefs = flow.reaching(i, "s", sb[2])
            ok_hi, saw_fence = fenced_scalar(flow, i, sb[2])
            if saw_fence or any(TILE_OR64.match(d) for d in bdefs):
                if not (ok_hi and fenced_scalar(flow, i, sb[1])[0]):
                    problems.append(f"{pretty}: tile access `{what}`: base also defined by {sorted(bdefs)}")
                for d in flow.reaching(i, "v", va[1]):
                    lit = LANE_CONFINED.match(d)
                    if not (ZERO_V.match(d) or (lit and int(lit.group(1), 0) < 4096)):
                        problems.append(f"{pretty}: tile access `{what}`: offset defined by `{d}`")
                tiles += 1
                continue
        if variant == 1:
            if not (va and va[0] == "v" and va[1] == va[2] and sb and sb[0] == "s"):
                problems.append(f"{pretty}: 32-bit fence but not SGPR-base + VGPR-offset: {what}")
                continue
            for d in flow.reaching(i, "v", va[1]):
                if not FENCE_AND32.match(d):
                    problems.append(f"{pretty}: offset {addr} of `{what}` defined by `{d}`")
        else:
            if not (va and va[0] == "v" and va[2] == va[1] + 1 and base == "off"):
                problems.append(f"{pretty}: 64-bit fence but not a 64-bit VGPR address: {what}")
                continue
            for d in flow.reaching(i, "v", va[2]):
                if not FENCE_OR32.match(d):
                    problems.append(f"{pretty}: high word v{va[2]} of `{what}` defined by `{d}`")
    if own_ws and variant in (1, 2) and own_ws_seen == 0:
        problems.append(f"{pretty}: expected an access to the library's own partial-sum array")
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
                # the measurement aids (k_*probe*) take no tenant and no fence: their template argument is not a rule
                variant = int(v.group(1)) if v and "probe" not in p else -1
                pr, ld, st, fc = lint_kernel(n, p, bodies[n], variant)
                md = meta.get(n, {})
                if md.get("scratch", 0) > 0:
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
