"""Coverage audit on the compiler's gfx950 assembly (no GPU needed: hipcc cross-compiles):
every global access of every fenced kernel carries the fence, no flat accesses,
no indirect branches, no scratch."""
import shutil

import pytest

from paper_2401_09290_amd import isa_lint


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_every_global_access_of_the_fenced_kernels_is_fenced():
    rows, problems, _ = isa_lint.run(verbose=False)
    assert not problems, "\n".join(problems)
    names = {r[0] for r in rows}
    # all six variants of every kernel; the DMA ring kernels for the four rules they are built for
    for v in range(6):
        assert f"k_stream<{v}, 1, true>" in names and f"k_stream<{v}, 1, false>" in names and f"k_gather32<{v}, 1>" in names and f"k_sum_partial<{v}, false>" in names
        assert {f"k_rmsnorm_bf16<{v}, 2, true>", f"k_rmsnorm_bf16<{v}, 2, false>", f"k_rmsnorm_bf16<{v}, 4, false>"} <= set(names) and f"k_gemm_nk256<{v}, true>" in names
    for v in range(4):
        assert f"k_gemm_ring<{v}, false>" in names
    # the per-array form of the modulo and checking rules, the buffer-load form of the hardware-checked rule
    for kern in ("k_gemm_ring", "k_gemm_units"):
        assert f"{kern}<3, true>" in names and f"{kern}<4, true>" in names and f"{kern}<5, false>" in names
    fenced = [r for r in rows if r[1] in (1, 2) and (r[2] + r[3]) > 0]
    assert fenced and all(r[4] > 0 for r in fenced if r[1] == 1)        # the 32-bit fence shows up as v_and_b32
    # the fence costs at most a handful of registers (the paper: up to two at -O3)
    base = {r[0].replace("<1", "<0", 1): r for r in rows if r[1] == 0}
    for r in rows:
        if r[1] == 1 and r[0].replace("<1", "<0", 1) in base and "gemm" not in r[0]:
            assert r[5] - base[r[0].replace("<1", "<0", 1)][5] <= 4, r



# ---- the audit itself, on hand-made assembly: a planted mistake must be reported ----------

GOOD_TILE = """
    s_load_dwordx4 s[4:7], s[0:1], 0x0
    v_and_b32 v1, 0x3ff, v0
    s_cmp_eq_u32 s2, 0
    s_cbranch_scc1 .LBB0_2
    s_and_b64 s[8:9], s[4:5], s[6:7]
    s_or_b64 s[8:9], s[8:9], s[10:11]
    s_branch .LBB0_3
.LBB0_2:
    s_and_b64 s[8:9], s[12:13], s[6:7]
    s_or_b64 s[8:9], s[8:9], s[10:11]
.LBB0_3:
    global_load_dwordx4 v[2:5], v1, s[8:9] nt
    s_endpgm
"""


def lint_text(text, variant):
    body = [ln.split(";")[0].rstrip() for ln in text.strip().splitlines()]
    return isa_lint.lint_kernel("k", "k_test<%d>" % variant, body, variant)[0]


def test_audit_follows_every_path_to_an_access():
    assert lint_text(GOOD_TILE, 2) == []
    # one of the two paths forgets the OR with the base: the base pair then has an unfenced definition
    bad = GOOD_TILE.replace("    s_and_b64 s[8:9], s[12:13], s[6:7]\n    s_or_b64 s[8:9], s[8:9], s[10:11]\n",
                            "    s_and_b64 s[8:9], s[12:13], s[6:7]\n")
    assert bad != GOOD_TILE
    assert any("base also defined" in p for p in lint_text(bad, 2))
    # a lane offset that is not confined below the tile size
    assert any("offset defined by" in p for p in lint_text(GOOD_TILE.replace("v_and_b32 v1, 0x3ff, v0", "v_lshlrev_b32 v1, 4, v0"), 2))
    # per-lane rules: an offset that skips the AND on one path (32-bit rule), a high word without the OR (64-bit rule)
    lane32 = """
    v_lshlrev_b32 v1, 2, v0
    s_cbranch_scc1 .LBB0_2
    v_and_b32 v1, s6, v1
.LBB0_2:
    global_store_dword v1, v2, s[4:5]
    s_endpgm
"""
    assert any("defined by `v_lshlrev_b32" in p for p in lint_text(lane32, 1))
    assert lint_text(lane32.replace("    s_cbranch_scc1 .LBB0_2\n", ""), 1) == []
    lane64 = """
    v_and_b32 v3, s7, v3
    v_or_b32 v3, s5, v3
    global_load_dword v4, v[2:3], off
    s_endpgm
"""
    assert lint_text(lane64, 2) == []
    assert lint_text(lane64.replace("    v_or_b32 v3, s5, v3\n", ""), 2)
    assert any("flat access" in p for p in lint_text("    flat_load_dword v1, v[2:3]\n    s_endpgm", 0))


def test_audit_follows_fenced_start_plus_offset_chains():
    """An array fenced once (s_and_b64 / s_or_b64 of its first byte) and then addressed as fenced start +
    offset, with the offset advanced by scalar adds inside a loop; the same chain from an unfenced start fails."""
    good = """
    v_and_b32 v1, 0x3ff, v0
    s_and_b64 s[8:9], s[4:5], s[6:7]
    s_or_b64 s[8:9], s[8:9], s[10:11]
    s_add_u32 s12, s8, s20
    s_addc_u32 s13, s9, s21
.LBB0_1:
    global_load_dwordx4 v[2:5], v1, s[12:13] offset:16 nt
    s_add_u32 s12, s12, s22
    s_addc_u32 s13, s13, s23
    s_cbranch_scc1 .LBB0_1
    s_endpgm
"""
    assert lint_text(good, 2) == []
    # the start is the raw pointer: no s_or_b64 anywhere in the chain -> the 64-bit rule's per-lane check rejects the access
    raw = good.replace("    s_and_b64 s[8:9], s[4:5], s[6:7]\n    s_or_b64 s[8:9], s[8:9], s[10:11]\n", "    s_mov_b64 s[8:9], s[4:5]\n")
    assert lint_text(raw, 2)
    # fenced low word but the high word of the sum comes from somewhere else
    mixed = good.replace("s_addc_u32 s13, s9, s21", "s_addc_u32 s13, s30, s21")
    assert lint_text(mixed, 2)
    # fenced high word, but the low word of the base comes from an unfenced register
    low = good.replace("s_add_u32 s12, s8, s20", "s_add_u32 s12, s30, s20")
    assert any("base also defined" in p for p in lint_text(low, 2))


def test_registers_of_a_load_in_flight_are_left_alone_until_a_wait_covers_it():
    """Hand-placed waits: between a load and the s_waitcnt vmcnt(k) that covers it (k at most the number of
    vector-memory instructions issued behind it) nothing may read or write its result registers."""
    good = """
    s_and_b64 s[8:9], s[4:5], s[6:7]
    s_or_b64 s[8:9], s[8:9], s[10:11]
    v_and_b32 v1, 0x3ff, v0
    global_load_dwordx4 v[2:5], v1, s[8:9]
    global_load_dwordx4 v[6:9], v1, s[8:9] offset:1024
    s_waitcnt vmcnt(1)
    v_add_f32 v10, v2, v3
    s_waitcnt vmcnt(0)
    v_add_f32 v10, v10, v6
    s_endpgm
"""
    pending = lambda text: [p for p in lint_text(text, 2) if "before a wait covers" in p]
    assert lint_text(good, 2) == []
    # the second load is read after a wait that only covers the first
    assert pending(good.replace("    s_waitcnt vmcnt(0)\n", ""))
    # a copy of the result registers placed before the wait: what a compiler that does not know of the load may do
    moved = good.replace("    s_waitcnt vmcnt(1)\n", "    v_mov_b32 v12, v3\n    s_waitcnt vmcnt(1)\n")
    assert moved != good and any("v_mov_b32 v12, v3" in p for p in pending(moved))
    # so is reusing one of them as a temporary
    assert pending(good.replace("    s_waitcnt vmcnt(1)\n", "    v_mov_b32 v4, 0\n    s_waitcnt vmcnt(1)\n"))
    # a store behind the loads shares the counter but completes in an order of its own: it can only make a wait
    # stricter, never stand for one of the instructions that may still be in flight
    store = good.replace("    s_waitcnt vmcnt(1)\n", "    global_store_dword v1, v11, s[8:9]\n    s_waitcnt vmcnt(1)\n")
    assert store != good and not pending(store)
    assert any("v_add_f32 v10, v2, v3" in p for p in pending(store.replace("vmcnt(1)", "vmcnt(2)")))
    # one path of two skips the wait
    branch = good.replace("    s_waitcnt vmcnt(1)\n", "    s_cbranch_scc1 .LBB0_1\n    s_waitcnt vmcnt(1)\n.LBB0_1:\n")
    assert any("v_add_f32 v10, v2, v3" in p for p in pending(branch))
    # a younger load into the same registers is in order (loads return in issue order); reading them before its own wait is not
    again = good.replace("    s_waitcnt vmcnt(1)\n", "    global_load_dwordx4 v[2:5], v1, s[8:9] offset:2048\n    s_waitcnt vmcnt(0)\n")
    assert lint_text(again, 2) == []
    assert pending(again.replace("    s_waitcnt vmcnt(0)\n    v_add_f32 v10, v2, v3", "    s_waitcnt vmcnt(1)\n    v_add_f32 v10, v2, v3"))
    # the numeric form of the wait is read as well: 0x0f70 is vmcnt(0) with the other counters open
    assert lint_text(good.replace("s_waitcnt vmcnt(0)", "s_waitcnt 0x0f70"), 2) == []


def test_data_registers_of_a_wide_store_are_left_alone_for_two_wait_states():
    """A store of more than 64 bits reads its data late: a vector-ALU write to those registers needs two wait
    states of distance.  The compiler pads its own stores; the hand-written ones carry an s_nop 1."""
    good = """
    s_and_b64 s[8:9], s[4:5], s[6:7]
    s_or_b64 s[8:9], s[8:9], s[10:11]
    v_and_b32 v1, 0x3ff, v0
    global_store_dwordx4 v1, v[2:5], s[8:9]
    s_nop 1
    v_mov_b32 v3, 0
    s_endpgm
"""
    hazard = lambda text: [p for p in lint_text(text, 2) if "within two wait states" in p]
    assert lint_text(good, 2) == []
    assert hazard(good.replace("    s_nop 1\n", ""))
    assert hazard(good.replace("    s_nop 1\n", "    s_nop 0\n"))
    assert not hazard(good.replace("    s_nop 1\n", "    s_mov_b32 s0, 0\n    s_mov_b32 s1, 0\n"))
    assert not hazard(good.replace("    s_nop 1\n", "").replace("v_mov_b32 v3, 0", "v_mov_b32 v6, 0"))        # other registers
    assert not hazard(good.replace("    s_nop 1\n", "").replace("dwordx4 v1, v[2:5]", "dwordx2 v1, v[2:3]"))   # 64 bits: no hazard
    # a load into the registers is no vector-ALU write
    assert not hazard(good.replace("    s_nop 1\n", "").replace("v_mov_b32 v3, 0", "global_load_dword v3, v1, s[8:9]\n    s_waitcnt vmcnt(0)"))


def test_scalar_registers_written_by_the_vector_alu_rest_five_wait_states_before_a_memory_instruction_reads_them():
    text = """
    v_readfirstlane_b32 s2, v1
    s_nop 3
    s_mov_b32 s3, 0
    global_load_dword v2, v0, s[2:3]
    s_waitcnt vmcnt(0)
    s_endpgm
"""
    hazard = lambda t: [p for p in lint_text(t, 0) if "fewer than five wait states" in p]
    assert not hazard(text)                                            # s_nop 3 = four wait states, plus the s_mov
    assert hazard(text.replace("s_nop 3", "s_nop 2"))
    assert hazard(text.replace("    s_nop 3\n", ""))
    assert not hazard(text.replace("    s_nop 3\n", "").replace("v_readfirstlane_b32 s2, v1", "s_mov_b32 s2, s9"))    # scalar writes are interlocked
    assert not hazard(text.replace("    s_nop 3\n", "").replace("v_readfirstlane_b32 s2, v1", "v_readfirstlane_b32 s6, v1"))
    # through a branch: the distance is counted along every path to the access
    branch = """
    v_cmp_lt_u32_e64 s[2:3], v1, v2
    s_cbranch_scc1 .LBB0_2
    s_nop 4
.LBB0_2:
    buffer_load_dword v2, v0, s[0:3], 0 offen
    s_waitcnt vmcnt(0)
    s_endpgm
"""
    assert hazard(branch) and not hazard(branch.replace("    s_cbranch_scc1 .LBB0_2\n", ""))


def test_m0_rests_one_wait_state_before_a_copy_to_the_lds():
    text = """
    s_and_b64 s[8:9], s[4:5], s[6:7]
    s_or_b64 s[8:9], s[8:9], s[10:11]
    v_and_b32 v1, 0x3ff, v0
    s_mov_b32 m0, s12
    s_nop 0
    global_load_lds_dwordx4 v1, s[8:9]
    s_waitcnt vmcnt(0)
    s_endpgm
"""
    hazard = lambda t: [p for p in lint_text(t, 2) if "M0 needs one wait state" in p]
    assert lint_text(text, 2) == []
    assert hazard(text.replace("    s_nop 0\n", ""))
    assert hazard(text.replace("    s_nop 0\n", "").replace("s_mov_b32 m0, s12", "s_add_u32 m0, s12, 16"))


# ---- dependency rules (all five rules), on real compiler output with planted mistakes -------

@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_planted_omissions_are_reported_in_every_rule(tmp_path):
    """tests/golden/isa_audit/planted.hip: one kernel that fences everything and four that forget the
    fence once each, built for the five rules.  The audit must report the forgetful ones, the access they
    forgot, and nothing else."""
    import os
    src = os.path.join(os.path.dirname(__file__), "golden", "isa_audit", "planted.hip")
    rows, problems = isa_lint.lint_file(src, str(tmp_path))
    assert len(rows) == 25
    by = {}
    for p in problems:
        by.setdefault(p.split(":")[0], []).append(p)
    for v in range(1, 6):
        assert f"k_planted_ok<{v}>" not in by, by.get(f"k_planted_ok<{v}>")
        raw = by.get(f"k_planted_raw_store<{v}>", [])
        assert raw and all("global_store_dword" in p for p in raw), (v, raw)
        uni = by.get(f"k_planted_uniform_read<{v}>", [])
        assert len(uni) == 1 and "scalar load from memory other than the kernel arguments" in uni[0], (v, uni)
        tile = by.get(f"k_planted_raw_tile<{v}>", [])
        if v == 5:      # any offset is bounded by the descriptor: nothing unsafe to report
            assert not tile, tile
        else:
            assert tile and all("global_load_dwordx4" in p for p in tile), (v, tile)
        wrong = by.get(f"k_planted_wrong_test<{v}>", [])
        if v == 4:      # tested against the other array's address: the store's own address met no comparison
            assert len(wrong) == 1 and "does not run under a comparison of its address" in wrong[0], wrong
        else:
            assert not wrong, wrong
    # the rule-specific dependency is what catches the modulo build (no instruction pattern is tied to that rule)
    assert any("does not depend on the fence's base, magic, size" in p for p in by["k_planted_raw_store<3>"])
    assert any("does not run under a comparison" in p for p in by["k_planted_raw_store<4>"])


# kernel arguments of the hand-made kernels below: pointer x at 0, pointer y at 8, then the fence's block at 16
# (base 16..23, size 24..31, reciprocal 32..39); explicit arguments end at 56
FO, END = 16, 56

CHECKED = """
    s_load_dwordx4 s[4:7], s[0:1], 0x0
    s_load_dwordx4 s[8:11], s[0:1], 0x10
    v_lshlrev_b32 v0, 2, v0
    v_mov_b32 v1, 0
    v_lshl_add_u64 v[2:3], s[4:5], 0, v[0:1]
    v_mov_b32 v6, s9
    v_subrev_co_u32 v4, vcc, s8, v2
    v_subb_co_u32 v5, vcc, v3, v6, vcc
    v_cmp_ge_u64 vcc, s[10:11], v[4:5]
    s_and_saveexec_b64 s[12:13], vcc
    s_xor_b64 s[12:13], exec, s[12:13]
    s_cbranch_execz .LBB0_2
    global_load_dword v7, v[2:3], off
.LBB0_2:
    s_andn2_saveexec_b64 s[12:13], s[12:13]
    s_cbranch_execz .LBB0_4
    global_atomic_add_x2 v1, v[8:9], s[14:15]
.LBB0_4:
    s_or_b64 exec, exec, s[12:13]
    s_endpgm
"""


def dep_problems(text, variant):
    body = [ln.split(";")[0].rstrip() for ln in text.strip().splitlines()]
    return isa_lint.lint_kernel("k", "k_test<%d>" % variant, body, variant, FO, END)[0]


def test_address_checking_regions_of_the_exec_mask():
    assert dep_problems(CHECKED, 4) == []
    # the load moved behind the point where the lanes that failed the comparison are switched back on
    late = CHECKED.replace("    global_load_dword v7, v[2:3], off\n", "").replace(
        "    s_or_b64 exec, exec, s[12:13]\n", "    s_or_b64 exec, exec, s[12:13]\n    global_load_dword v7, v[2:3], off\n")
    assert any("does not run under a comparison" in p for p in dep_problems(late, 4))
    # the comparison uses the other array's pointer: it does not cover what this address is made from
    other = CHECKED.replace("v_subrev_co_u32 v4, vcc, s8, v2", "v_subrev_co_u32 v4, vcc, s8, v10").replace(
        "v_subb_co_u32 v5, vcc, v3, v6, vcc", "v_subb_co_u32 v5, vcc, v11, v6, vcc").replace(
        "    v_mov_b32 v6, s9\n", "    v_mov_b32 v6, s9\n    v_lshl_add_u64 v[10:11], s[6:7], 0, v[0:1]\n")
    assert other != CHECKED and any("does not run under a comparison" in p for p in dep_problems(other, 4))
    # the comparison is against something that is not the partition's size
    nosize = CHECKED.replace("v_cmp_ge_u64 vcc, s[10:11], v[4:5]", "v_cmp_ge_u64 vcc, s[6:7], v[4:5]")
    assert any("does not run under a comparison" in p for p in dep_problems(nosize, 4))
    # an access in the second half of a two-way split is selected by the same comparison (its sense is the parity tests' matter)
    second = CHECKED.replace("global_atomic_add_x2 v1, v[8:9], s[14:15]", "global_load_dword v7, v[2:3], off")
    assert dep_problems(second, 4) == []
    # a whole-array test decided by a scalar branch
    branch = """
    s_load_dwordx4 s[4:7], s[0:1], 0x0
    s_load_dwordx4 s[8:11], s[0:1], 0x10
    s_sub_u32 s12, s4, s8
    s_subb_u32 s13, s5, s9
    v_mov_b64 v[2:3], s[12:13]
    v_cmp_ge_u64 vcc, s[10:11], v[2:3]
    s_cbranch_vccz .LBB0_2
    v_and_b32 v1, 0x3ff, v0
    global_load_dwordx4 v[4:7], v1, s[4:5]
.LBB0_2:
    s_endpgm
"""
    assert dep_problems(branch, 4) == []
    # ... but a branch both of whose outcomes run the access decides nothing
    both = branch.replace(".LBB0_2:\n", "").replace("    v_and_b32 v1, 0x3ff, v0\n", ".LBB0_2:\n    v_and_b32 v1, 0x3ff, v0\n")
    assert any("does not run under a comparison" in p for p in dep_problems(both, 4))


def test_modulo_rule_needs_base_size_and_reciprocal_in_every_address():
    good = """
    s_load_dwordx2 s[4:5], s[0:1], 0x0
    s_load_dwordx4 s[8:11], s[0:1], 0x10
    s_load_dwordx2 s[12:13], s[0:1], 0x20
    v_lshlrev_b32 v0, 2, v0
    v_mov_b32 v1, 0
    v_lshl_add_u64 v[2:3], s[4:5], 0, v[0:1]
    v_subrev_co_u32 v4, vcc, s8, v2
    v_mul_hi_u32 v5, s12, v4
    v_mul_lo_u32 v5, v5, s10
    v_sub_u32 v4, v4, v5
    v_mov_b32 v5, 0
    v_lshl_add_u64 v[6:7], s[8:9], 0, v[4:5]
    global_load_dword v8, v[6:7], off
    s_endpgm
"""
    assert dep_problems(good, 3) == []
    raw = good.replace("global_load_dword v8, v[6:7], off", "global_load_dword v8, v[2:3], off")
    assert any("does not depend on the fence's base, magic, size" in p for p in dep_problems(raw, 3))
    # base added, but the remainder was never taken
    noq = good.replace("    v_mul_hi_u32 v5, s12, v4\n    v_mul_lo_u32 v5, v5, s10\n    v_sub_u32 v4, v4, v5\n", "")
    assert any("does not depend on the fence's magic, size" in p for p in dep_problems(noq, 3))
    # the bitwise rules: an AND with a scalar that is not the partition's mask
    lane32 = """
    s_load_dwordx2 s[4:5], s[0:1], 0x0
    s_load_dwordx4 s[8:11], s[0:1], 0x10
    v_lshlrev_b32 v1, 2, v0
    v_add_u32 v1, s4, v1
    v_and_b32 v1, s10, v1
    global_store_dword v1, v2, s[8:9]
    s_endpgm
"""
    assert dep_problems(lane32, 1) == []
    assert any("does not depend on the fence's size" in p for p in dep_problems(lane32.replace("v_and_b32 v1, s10, v1", "v_and_b32 v1, s5, v1"), 1))
    # scalar loads: kernel arguments only (also through the pointer plus a constant)
    assert dep_problems("    s_add_u32 s6, s0, 0x50\n    s_addc_u32 s7, s1, 0\n    s_load_dword s2, s[6:7], 0x0\n    s_endpgm", 0) == []
    assert any("scalar load from memory other than the kernel arguments" in p
               for p in dep_problems("    s_load_dwordx2 s[4:5], s[0:1], 0x0\n    s_load_dword s2, s[4:5], 0x0\n    s_endpgm", 0))
