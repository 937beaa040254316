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
* for all five rules, on the backward slice of each access's address registers (through
  registers, condition codes and earlier loads, down to the scalar loads of the kernel
  arguments, whose layout the code object's metadata gives): scalar loads read the kernel
  arguments only; under the bitwise and hardware-checked rules every address depends on the
  partition's base and size, under the modulo rule also on the reciprocal; under address
  checking every access runs under a scalar branch or an exec-mask selection that depends on
  base, size and on every kernel argument its own address depends on.  This shows that no
  access bypasses its rule; that the rule's arithmetic and the comparison's sense are right
  is what the parity tests show (images, neighbours' bytes, exact fault counts);
* in every kernel (some loads, stores and waits are written by hand, and the compiler neither counts
  nor pads those): no instruction names the result registers of a vector-memory load before an
  s_waitcnt vmcnt covers that load; no vector-ALU write to the data registers of a 128-bit store
  within two wait states; five wait states between a vector-ALU write to a scalar register and a
  vector-memory instruction that reads it; one wait state between a write of M0 and a global -> LDS copy;
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


def fence_param_index(mangled):
    """Position of the gd::FenceArgs parameter in a kernel's parameter list, read off the Itanium name
    (parameters here are structs passed by value, pointers and builtin integers), or None."""
    m = re.match(r"^_ZN2gd\d+[a-z_0-9]+?(?:I.*?E)?Ev(.*)$", mangled)
    if not m:
        return None
    rest, k = m.group(1), 0
    while rest:
        rest = rest.lstrip("PK")
        if rest.startswith("NS_9FenceArgsE"):
            return k
        nested = rest.startswith("N")
        rest = rest[1:] if nested else rest
        parts = 0
        while True:
            d = re.match(r"^(\d+)", rest)
            sub = re.match(r"^S[0-9A-Z]*_", rest)
            if d:
                rest = rest[len(d.group(1)) + int(d.group(1)):]
            elif sub:
                rest = rest[sub.end():]
            else:
                break
            parts += 1
            if not nested:
                break
        if nested:
            if not rest.startswith("E"):
                return None
            rest = rest[1:]
        elif parts == 0:
            if not rest or not rest[0].isalpha():
                return None
            rest = rest[1:]                              # a builtin type
        k += 1
    return None


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
    # kernel arguments from the code object's metadata; which of them is the fence's 40-byte parameter block
    # follows from the position of gd::FenceArgs in the kernel's (mangled) parameter list
    for m in re.finditer(r"\.args:\n(.*?)\n    \.group_segment_fixed_size.*?\.name:\s+(\S+)", asm_text, re.S):
        args = re.findall(r"\.offset:\s+(\d+)\n\s+\.size:\s+(\d+)\n\s+\.value_kind:\s+(\w+)", m.group(1))
        explicit = [(int(o), int(z)) for o, z, kind in args if not kind.startswith("hidden")]
        if m.group(2) in meta and explicit:
            meta[m.group(2)]["explicit_end"] = explicit[-1][0] + explicit[-1][1]
            k = fence_param_index(m.group(2))
            meta[m.group(2)]["fence_offset"] = explicit[k][0] if k is not None and k < len(explicit) and explicit[k][1] == 40 else None
    return bodies, meta


NO_DEST = ("s_cmp", "s_cbranch", "s_branch", "s_waitcnt", "s_barrier", "s_nop", "s_endpgm", "s_setprio", "s_sleep",
           "s_bitcmp", "s_setreg", "s_sendmsg", "s_trap", "global_store", "ds_write", "buffer_store",
           "global_load_lds", "v_cmpx", "v_nop", "s_mov_b32 m0")
# instructions whose second operand is written as well (carry / scale outputs)
TWO_DEST = ("v_mad_u64_u32", "v_mad_i64_i32", "v_add_co_u32", "v_sub_co_u32", "v_subrev_co_u32", "v_addc_co_u32",
            "v_subb_co_u32", "v_subbrev_co_u32", "v_div_scale_f32", "v_div_scale_f64")
# condition registers, tracked as kind 'x': vcc, scc, exec (halves count as the whole)
SPECIAL = {"vcc": 0, "vcc_lo": 0, "vcc_hi": 0, "scc": 1, "exec": 2, "exec_lo": 2, "exec_hi": 2}
VCC, SCC, EXEC = ("x", 0, 0), ("x", 1, 1), ("x", 2, 2)
# scalar instructions that leave their outcome in scc
SCC_WRITERS = ("s_add_", "s_addc_", "s_sub_", "s_subb_", "s_and_", "s_andn2_", "s_or_", "s_orn2_", "s_xor_", "s_nand_",
               "s_nor_", "s_xnor_", "s_lshl_", "s_lshr_", "s_ashr_", "s_bfe_", "s_cmp_", "s_bitcmp", "s_min_", "s_max_",
               "s_abs_", "s_not_", "s_bcnt", "s_absdiff", "s_lshl1_add", "s_lshl2_add", "s_lshl3_add", "s_lshl4_add",
               "s_wqm", "s_quadmask")
SCC_READERS = ("s_addc_", "s_subb_", "s_cselect", "s_cmov", "s_cbranch_scc")


def _regs(operand):
    """('v'|'s'|'x', lo, hi) of a register operand, or None."""
    operand = operand.lstrip("-|").rstrip("|")
    m = re.match(r"^([vs])(\d+)$", operand)
    if m:
        return m.group(1), int(m.group(2)), int(m.group(2))
    m = re.match(r"^([vs])\[(\d+):(\d+)\]$", operand)
    if m:
        return m.group(1), int(m.group(2)), int(m.group(3))
    if operand in SPECIAL:
        return "x", SPECIAL[operand], SPECIAL[operand]
    return None


def _split(line):
    code = line.strip()
    m = re.match(r"^(\w+)\s*(.*)$", code)
    if not m or LABEL_RE.match(code):
        return None, []
    return m.group(1), [o.strip().split()[0] for o in m.group(2).split(",") if o.strip()]


def _no_return_atomic(op, ops):
    """global_atomic_* vaddr, vdata, saddr (three operands): nothing comes back, nothing is written."""
    return op.startswith("global_atomic") and len(ops) == 3


def dests(line):
    """Registers an instruction writes: its explicit results, and scc / exec where the
    instruction leaves its outcome there (m0 is not tracked)."""
    op, ops = _split(line)
    if op is None:
        return []
    out = []
    if not line.strip().startswith(NO_DEST) and not _no_return_atomic(op, ops):
        for k in range(2 if op.startswith(TWO_DEST) else 1):
            if k < len(ops) and _regs(ops[k]):
                out.append(_regs(ops[k]))
    if op.startswith(SCC_WRITERS):
        out.append(SCC)
    if "saveexec" in op or op.startswith("v_cmpx"):
        out.append(EXEC)
    return out


def srcs(line):
    """Registers an instruction reads (explicit operands, and scc / vcc / exec where a
    branch, a carry or an exec-mask update takes them implicitly)."""
    op, ops = _split(line)
    if op is None:
        return []
    if (line.strip().startswith(NO_DEST) and not line.strip().startswith("s_mov_b32 m0")) or _no_return_atomic(op, ops):
        first = 0
    else:
        first = 2 if op.startswith(TWO_DEST) else 1
    out = [r for r in (_regs(o) for o in ops[first:]) if r]
    if op.startswith(SCC_READERS):
        out.append(SCC)
    if op.startswith("s_cbranch_vcc"):
        out.append(VCC)
    if op.startswith("s_cbranch_exec") or "saveexec" in op:
        out.append(EXEC)
    return out


class Flow:
    """Control-flow graph of one kernel body; reaching definitions, dominators and
    backward slices on it."""

    def __init__(self, body):
        self.body = body
        n = len(body)
        label_at = {}
        for i, ln in enumerate(body):
            m = LABEL_RE.match(ln.strip())
            if m:
                label_at[m.group(1)] = i
        self.preds = [[] for _ in range(n + 1)]            # instruction index -> indices it can be reached from
        self.succs = [[] for _ in range(n + 1)]
        self.ops = []
        for i, ln in enumerate(body):
            code = ln.strip()
            op = code.split()[0] if code else ""
            self.ops.append(op)
            target = code.split()[-1] if op.startswith(("s_branch", "s_cbranch")) else None
            if target is not None and target in label_at:
                self.preds[label_at[target]].append(i)
                self.succs[i].append(label_at[target])
            if not op.startswith(("s_branch", "s_endpgm")) and i + 1 < n:
                self.preds[i + 1].append(i)
                self.succs[i].append(i + 1)
        self.dst = [dests(ln) for ln in body]
        self._dom = None
        self._reach = {}                                   # memo of reaching_at

    def reaching_at(self, idx, kind, reg):
        """Indices of the instructions whose write of `reg` can reach instruction idx; -1 stands for
        the value the register holds when the kernel starts."""
        key = (idx, kind, reg)
        if key in self._reach:
            return self._reach[key]
        found, seen, stack = set(), set(), list(self.preds[idx])
        if not stack:
            found.add(-1)
        self._reach[key] = found
        while stack:
            j = stack.pop()
            if j in seen:
                continue
            seen.add(j)
            if any(k == kind and lo <= reg <= hi for (k, lo, hi) in self.dst[j]):
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

    def dominators(self, idx):
        """Indices of the instructions every path from the kernel's start to idx passes (idx included),
        as a bit set in a Python integer."""
        if self._dom is None:
            n = len(self.body)
            full = (1 << n) - 1
            dom = [full] * n
            if n:
                dom[0] = 1
            changed = True
            while changed:
                changed = False
                for i in range(1, n):
                    acc = full
                    for p in self.preds[i]:
                        acc &= dom[p]
                    if not self.preds[i]:
                        acc = 0                            # unreachable text
                    acc |= 1 << i
                    if acc != dom[i]:
                        dom[i], changed = acc, True
            self._dom = dom
        return self._dom[idx]

    def slice_of(self, idx, regs, through_exec=True):
        """Backward slice: every instruction whose result can flow into one of `regs`
        (a list of (kind, number)) as read by instruction idx.  Returns {(j, kind, number)}: definition j
        (-1 = kernel start) was reached for that register.  through_exec=False does not follow the exec
        mask an exec-mask update read (the conditions that were already in force), only what it combined
        it with."""
        out, seen = set(), set()
        work = [(idx, k, r) for (k, r) in regs]
        while work:
            i, k, r = work.pop()
            if (i, k, r) in seen:
                continue
            seen.add((i, k, r))
            for j in self.reaching_at(i, k, r):
                out.add((j, k, r))
                if j >= 0:
                    for (sk, lo, hi) in srcs(self.body[j]):
                        if (sk, lo, hi) == EXEC and not through_exec:
                            continue
                        for q in range(lo, hi + 1):
                            work.append((j, sk, q))
        return out

    def reaches_end_avoiding(self, start, avoid):
        """Can the kernel end, starting at instruction `start`, without executing instruction `avoid`?"""
        seen, stack = set(), [start]
        while stack:
            j = stack.pop()
            if j in seen or j == avoid:
                continue
            seen.add(j)
            if self.ops[j].startswith("s_endpgm") or not self.succs[j]:
                return True
            stack.extend(self.succs[j])
        return False


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


LOAD_BYTES = {"s_load_dword": 4, "s_load_dwordx2": 8, "s_load_dwordx4": 16, "s_load_dwordx8": 32, "s_load_dwordx16": 64}
FENCE_FIELDS = {"base": (0, 8), "size": (8, 16), "magic": (16, 24)}      # byte ranges inside the fence's kernel parameter
NEEDS = {1: ("base", "size"), 2: ("base", "size"), 3: ("base", "size", "magic"), 5: ("base", "size")}
# exec-mask updates that select lanes by a condition: "then" (AND with the condition), loop exits, and the "else"
# half of a two-way split (saved mask AND NOT the lanes that ran the first half)
EXEC_NARROW = re.compile(r"^(s_and_saveexec_b64\s|s_and_b64\s+exec,|s_andn2_b64\s+exec,\s*exec,|s_andn2_saveexec_b64\s)")
EXEC_WIDEN = re.compile(r"^(s_or_b64\s+exec,|s_mov_b64\s+exec,|s_xor_b64\s+exec,|s_andn2_saveexec_b64\s|s_or_saveexec_b64\s|"
                        r"s_xor_saveexec_b64\s|s_orn2_saveexec_b64\s|s_andn2_wrexec)")
MASK_ALGEBRA = ("s_and_b64", "s_or_b64", "s_xor_b64", "s_andn2_b64", "s_mov_b64")


def mask_within(flow, idx, pair, guard, depth=0, seen=None):
    """Is the lane mask in the SGPR pair `pair` = (lo, hi), as read by instruction idx, a subset of the
    exec mask that the narrowing instruction `guard` left?  True for masks saved from exec inside the
    guard's region and for combinations of such masks with exec; false for the mask the guard itself
    saved (the lanes in force before it) and for anything else."""
    seen = set() if seen is None else seen
    if depth > 8:
        return False
    for d in flow.reaching_at(idx, "s", pair[0]) | flow.reaching_at(idx, "s", pair[1]):
        if d < 0 or d == guard or not (flow.dominators(d) >> guard) & 1:
            return False
        if (d, pair) in seen:
            continue
        seen.add((d, pair))
        op, ops = _split(flow.body[d])
        if "saveexec" in op:
            continue                                       # exec as it stood at d, inside the region
        if not op.startswith(MASK_ALGEBRA):
            return False
        for o in ops[1:]:
            r = _regs(o)
            if r == EXEC:
                continue
            if not (r and r[0] == "s" and r[2] == r[1] + 1 and mask_within(flow, d, (r[1], r[2]), guard, depth + 1, seen)):
                return False
    return True


def widens(flow, k, guard):
    """Does instruction k (an exec-mask update) let lanes run that the narrowing `guard` switched off?"""
    text = flow.body[k].strip()
    if not EXEC_WIDEN.match(text):
        return False
    op, ops = _split(text)
    for o in ops[1:]:
        r = _regs(o)
        if r == EXEC:
            continue
        if not (r and r[0] == "s" and r[2] == r[1] + 1 and mask_within(flow, k, (r[1], r[2]), guard)):
            return True
    return False


def kernarg_offset(flow, idx, lo, hi):
    """If the SGPR pair s[lo:hi], as read by instruction idx, is the kernel-argument pointer the kernel
    starts with in s[0:1], or that pointer plus a constant, return the constant; otherwise None."""
    dl, dh = flow.reaching_at(idx, "s", lo), flow.reaching_at(idx, "s", hi)
    if dl == {-1} and dh == {-1}:
        return 0 if (lo, hi) == (0, 1) else None
    if len(dl) == 1 and len(dh) == 1:
        jl, jh = next(iter(dl)), next(iter(dh))
        if jl >= 0 and jh >= 0:
            ml = re.match(r"^s_add_u32\s+s\d+,\s*s0,\s*(0x[0-9a-f]+|\d+)$", flow.body[jl].strip())
            mh = re.match(r"^s_addc_u32\s+s\d+,\s*s1,\s*0$", flow.body[jh].strip())
            if ml and mh and flow.reaching_at(jl, "s", 0) == {-1} and flow.reaching_at(jh, "s", 1) == {-1}:
                return int(ml.group(1), 0)
    return None


def scalar_load(flow, j):
    """(first result SGPR, kernel-argument byte offset or None) of the scalar load at instruction j."""
    op, ops = _split(flow.body[j])
    dst, base = _regs(ops[0]), _regs(ops[1])
    imm = int(ops[2], 0) if len(ops) > 2 and re.match(r"^(0x[0-9a-f]+|\d+)$", ops[2]) else None
    ko = kernarg_offset(flow, j, base[1], base[2]) if base and base[0] == "s" and base[2] == base[1] + 1 else None
    return dst[1], (ko + imm if ko is not None and imm is not None else None)


def kernarg_bytes(flow, sl):
    """Kernel-argument byte offsets (one per 4-byte word) that a backward slice depends on; None stands
    for a scalar load from anywhere else."""
    out = set()
    for (j, kind, reg) in sl:
        if j >= 0 and kind == "s" and flow.ops[j] in LOAD_BYTES:
            first, off = scalar_load(flow, j)
            out.add(None if off is None else off + 4 * (reg - first))
    return out


def fence_fields(words, fence_offset):
    return {name for name, (lo, hi) in FENCE_FIELDS.items() if any(w is not None and fence_offset + lo <= w < fence_offset + hi for w in words)}


def guarded_by_bounds(flow, i, addr_words, fence_offset):
    """Address checking: is the access at instruction i executed only under a condition that depends on the
    partition's base and size and on everything its own address depends on?  The condition is a scalar
    branch that decides whether i runs, or an exec-mask narrowing that still holds at i."""
    dom = flow.dominators(i)
    for j in range(i - 1, -1, -1):
        if not (dom >> j) & 1:
            continue
        op, text = flow.ops[j], flow.body[j].strip()
        if op.startswith(("s_cbranch_scc", "s_cbranch_vcc")):
            if not flow.reaches_end_avoiding(j, i):
                continue                                  # both outcomes run the access: it does not depend on this branch
            cond = [("x", SCC[1] if "scc" in op else VCC[1])]
        elif EXEC_NARROW.match(text):
            seen, stack, widened = set(), list(flow.preds[i]), False
            while stack and not widened:                  # every path from the narrowing to the access: no widening on it
                k = stack.pop()
                if k in seen or k == j:
                    continue
                seen.add(k)
                widened = widens(flow, k, j)
                stack.extend(flow.preds[k])
            if widened:
                continue
            cond = [(k, q) for (k, lo, hi) in srcs(text) for q in range(lo, hi + 1) if (k, lo, hi) != EXEC]
        else:
            continue
        words = kernarg_bytes(flow, flow.slice_of(j, cond, through_exec=False))
        if {"base", "size"} <= fence_fields(words, fence_offset) and addr_words <= words:
            return True
    return False


def access_address(line):
    """The registers that address a global or buffer access, as [(kind, number)], or None for other lines."""
    m = MEM_RE.match(line)
    if m:
        inst, ops = m.group(1), [o.strip().split()[0] for o in m.group(2).split(",")]
        if inst.startswith("global_load_lds"):
            parts = ops[0:2]
        elif inst.startswith("global_store"):
            parts = [ops[0]] + ops[2:3]
        elif inst.startswith("global_atomic") and len(ops) == 3:     # no returned value: address, data, base
            parts = [ops[0], ops[2]]
        else:
            parts = ops[1:3]
    else:
        m = BUF_RE.match(line)
        if not m:
            return None
        inst, ops = m.group(1), [o.strip().split()[0] for o in m.group(2).split(",")]
        parts = ops[1:4]                                           # offset VGPR, descriptor, scalar offset
    return inst, [(r[0], q) for r in (_regs(o) for o in parts) if r for q in range(r[1], r[2] + 1)]


def dependency_problems(flow, pretty, variant, fence_offset, explicit_end, own_ws=False):
    """What each access's address is computed from, on the backward slice of its address registers.

    * No scalar load reads anything but the kernel arguments (tenant memory is never read through the
      scalar cache, where no rule applies).
    * Bitwise, modulo and hardware-checked rules: the address of every access to tenant memory depends on
      the partition's base and size (and, modulo rule, on the reciprocal): an address that never met the
      fence cannot.
    * Address checking: every access runs under a condition (guarded_by_bounds) that depends on base, size
      and on every kernel argument the address itself depends on.
    This shows that no access bypasses the rule; that the rule's arithmetic and the comparison's sense are
    right is what the parity tests show (images, neighbours' bytes, exact fault counts)."""
    problems = []
    for i, ln in enumerate(flow.body):
        if flow.ops[i].startswith(("s_load_", "s_buffer_load")):
            if flow.ops[i] not in LOAD_BYTES or scalar_load(flow, i)[1] is None:
                problems.append(f"{pretty}: scalar load from memory other than the kernel arguments: {ln.strip()}")
            continue
        if fence_offset is None or variant not in (1, 2, 3, 4, 5):
            continue
        acc = access_address(ln)
        if acc is None or acc[0] in UNFENCED_OK:
            continue
        inst, regs = acc
        if own_ws and (("store" in inst and "k_sum_partial" in pretty) or ("load" in inst and "k_sum_final" in pretty)):
            continue                                      # the library's own partial-sum array
        words = kernarg_bytes(flow, flow.slice_of(i, regs))
        if variant == 4:
            # the tenant's argument block is what precedes the fence's parameters; what the library appends behind them
            # (launch geometry) is the manager's own
            mine = {w for w in words if w is not None and w < fence_offset}
            if not guarded_by_bounds(flow, i, mine, fence_offset):
                problems.append(f"{pretty}: `{ln.strip()}` does not run under a comparison of its address with the partition's bounds")
        else:
            missing = set(NEEDS[variant]) - fence_fields(words, fence_offset)
            if missing:
                problems.append(f"{pretty}: address of `{ln.strip()}` does not depend on the fence's {', '.join(sorted(missing))}")
    return problems


VMEM_LOAD = re.compile(r"^(global_load|buffer_load|flat_load)")
VMEM_LOAD_TO_REG = re.compile(r"^(global_load_(?!lds)|buffer_load_)")


def vmcnt_of(text):
    """The vmcnt a wait instruction asks for (gfx9 encoding of the numeric form), or None if it does not wait on it."""
    m = re.match(r"^s_waitcnt\s+(.*)$", text)
    if not m:
        return None
    arg = m.group(1).strip()
    v = re.search(r"vmcnt\((\d+)\)", arg)
    if v:
        return int(v.group(1))
    if re.match(r"^(0x[0-9a-f]+|\d+)$", arg):
        imm = int(arg, 0)
        return (imm & 0xF) | ((imm >> 14) & 0x3) << 4
    return None


def pending_load_problems(flow, pretty):
    """No instruction reads or writes the result registers of a vector-memory load before a wait covers it.

    The kernels place some waits by hand (Fence::ld_tile16 / tile_wait): the compiler does not know that the
    result registers of such a load are still in flight and may copy or reuse them.  From every load to
    registers the audit walks every path forward, counting the loads issued behind it, until an
    s_waitcnt vmcnt(k) with k not above that count: loads complete in issue order, so with the load still in
    flight more than k instructions would be outstanding.  Stores share the counter but complete in an order of
    their own, so a store behind the load does not count.  Any instruction met before that which names one of
    the load's result registers is reported, except a younger load that only writes them."""
    problems = []
    waits = [vmcnt_of(ln.strip()) for ln in flow.body]
    cap = max([k for k in waits if k is not None], default=0) + 1     # counts above every wait are alike
    for i, ln in enumerate(flow.body):
        text = ln.strip()
        if not VMEM_LOAD_TO_REG.match(text) or re.search(r"\blds\b", text):
            continue
        dst = flow.dst[i]
        if not dst:
            continue
        kind, lo, hi = dst[0]
        seen, stack = set(), [(s_, 0) for s_ in flow.succs[i]]
        while stack:
            j, younger = stack.pop()
            if (j, younger) in seen:
                continue
            seen.add((j, younger))
            t = flow.body[j].strip()
            k = waits[j]
            if k is not None and k <= younger:
                continue                                  # the load has landed on this path
            over = lambda regs: [r for r in regs if r[0] == kind and not (r[2] < lo or r[1] > hi)]
            # A younger load may take the same result registers: loads return in issue order, so the older
            # result (which nothing has read on this path) is overwritten by the younger one, never the reverse.
            younger_load = VMEM_LOAD_TO_REG.match(t) and not over(srcs(t))
            touched = over(srcs(t)) if younger_load else over(flow.dst[j] + srcs(t))
            if touched and not LABEL_RE.match(t):
                problems.append(f"{pretty}: `{t}` touches v[{lo}:{hi}] of `{text}` before a wait covers the load")
                continue
            if flow.ops[j].startswith("s_endpgm"):
                continue
            nxt = min(younger + 1, cap) if VMEM_LOAD.match(t) else younger
            stack.extend((s_, nxt) for s_ in flow.succs[j])
    return problems


WIDE_STORE = re.compile(r"^(global_store_dwordx[34]|buffer_store_dwordx[34]|flat_store_dwordx[34])\b")


def store_data_problems(flow, pretty):
    """No vector-ALU instruction overwrites the data registers of a store of more than 64 bits in the two
    wait states behind it (the store reads its data late; the compiler pads its own stores, but it cannot
    see the ones written as inline assembly)."""
    problems = []
    for i, ln in enumerate(flow.body):
        text = ln.strip()
        if not WIDE_STORE.match(text):
            continue
        op, ops = _split(text)
        data = _regs(ops[0]) if op.startswith("buffer_store") else _regs(ops[1])
        if not data or data[0] != "v":
            continue
        stack, seen = [(s_, 2) for s_ in flow.succs[i]], set()
        while stack:
            j, left = stack.pop()
            if left <= 0 or (j, left) in seen:
                continue
            seen.add((j, left))
            t = flow.body[j].strip()
            if LABEL_RE.match(t):
                stack.extend((s_, left) for s_ in flow.succs[j])
                continue
            if t.startswith("v_") and any(r[0] == "v" and not (r[2] < data[1] or r[1] > data[2]) for r in flow.dst[j]):
                problems.append(f"{pretty}: `{t}` overwrites the data of `{text}` within two wait states")
            m = re.match(r"^s_nop\s+(\d+)", t)
            spent = int(m.group(1)) + 1 if m else 1
            stack.extend((s_, left - spent) for s_ in flow.succs[j])
    return problems


VMEM_ANY = re.compile(r"^(global_|buffer_|flat_)(load|store|atomic)")


def sgpr_hazard_problems(flow, pretty):
    """A vector-memory instruction that reads a scalar register written by the vector ALU (v_readfirstlane,
    a comparison into a register pair, a carry-out) needs five wait states between the two.  The compiler
    keeps that distance for its own instructions; the audit checks it for all, the hand-written ones included."""
    problems = []
    for i, ln in enumerate(flow.body):
        text = ln.strip()
        if not VMEM_ANY.match(text):
            continue
        used = [r for r in srcs(text) if r[0] == "s"]
        if not used:
            continue
        stack, seen = [(j, 5) for j in flow.preds[i]], set()
        while stack:
            j, left = stack.pop()
            if left <= 0 or (j, left) in seen:
                continue
            seen.add((j, left))
            t = flow.body[j].strip()
            if LABEL_RE.match(t):
                stack.extend((k, left) for k in flow.preds[j])
                continue
            if t.startswith("v_") and any(d[0] == "s" and any(not (d[2] < u[1] or d[1] > u[2]) for u in used) for d in flow.dst[j]):
                problems.append(f"{pretty}: `{text}` reads a scalar register that `{t}` wrote fewer than five wait states earlier")
                continue
            m = re.match(r"^s_nop\s+(\d+)", t)
            spent = int(m.group(1)) + 1 if m else 1
            stack.extend((k, left - spent) for k in flow.preds[j])
    return problems


LDS_DMA = re.compile(r"^(global_load_lds_|buffer_load_\S+ .*\blds\b)")


def m0_hazard_problems(flow, pretty):
    """A global -> LDS copy takes its LDS address from M0: one wait state between the scalar write of M0 and
    the copy (the hand-written copies carry an s_nop 0)."""
    problems = []
    for i, ln in enumerate(flow.body):
        text = ln.strip()
        if not LDS_DMA.match(text):
            continue
        for j in flow.preds[i]:
            t = flow.body[j].strip()
            if re.match(r"^s_\w+\s+m0\b", t):
                problems.append(f"{pretty}: `{text}` directly behind `{t}`: M0 needs one wait state")
    return problems


def lint_kernel(name, pretty, body, variant, fence_offset=None, explicit_end=None):
    """fence_offset / explicit_end: byte offset of the fence's parameter block among the kernel arguments and
    the end of the explicit arguments (from the code object's metadata); the dependency rules need them."""
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
    if variant >= 0:
        problems += dependency_problems(flow, pretty, variant, fence_offset, explicit_end, own_ws)
    problems += pending_load_problems(flow, pretty)
    problems += store_data_problems(flow, pretty)
    problems += sgpr_hazard_problems(flow, pretty)
    problems += m0_hazard_problems(flow, pretty)
    return problems, loads, stores, fences


def lint_file(source, tmp):
    """Compile one HIP source to gfx950 assembly and audit every gd:: kernel in it.
    Returns (rows, problems); a row is (kernel, variant, loads, stores, fences, VGPRs, SGPRs, scratch)."""
    rows, problems = [], []
    out = os.path.join(tmp, os.path.basename(source) + ".s")
    res = subprocess.run(["hipcc", *FLAGS, "-o", out, source], capture_output=True, text=True)
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
        md = meta.get(n, {})
        pr, ld, st, fc = lint_kernel(n, p, bodies[n], variant, md.get("fence_offset"), md.get("explicit_end"))
        if variant > 0 and md.get("fence_offset") is None:
            pr.append(f"{p}: the fence's parameter block was not found among the kernel arguments")
        if md.get("scratch", 0) > 0:
            pr.append(f"{p}: uses {md['scratch']} bytes of scratch")
        problems += pr
        rows.append((p, variant, ld, st, fc, md.get("vgpr", -1), md.get("sgpr", -1), md.get("scratch", -1)))
    return rows, problems


def run(verbose=True):
    rows, problems = [], []
    with tempfile.TemporaryDirectory() as tmp:
        for src in HIP_SOURCES:
            r, pr = lint_file(os.path.join(CSRC, src), tmp)
            rows += r
            problems += pr
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
