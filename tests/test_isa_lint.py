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
        assert f"k_rmsnorm_bf16<{v}>" in names and f"k_gemm_nk256<{v}, true>" in names
    for v in range(4):
        assert f"k_gemm_ring<{v}>" in names
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
