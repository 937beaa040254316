"""Coverage audit on the compiler's gfx950 assembly (no GPU needed: hipcc cross-compiles):
every global access of every fenced kernel carries the fence, no flat accesses,
no indirect branches, no scratch outside the GEMM."""
import shutil

import pytest

from paper_2401_09290_amd import isa_lint


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_every_global_access_of_the_fenced_kernels_is_fenced():
    rows, problems, _ = isa_lint.run(verbose=False)
    assert not problems, "\n".join(problems)
    names = {r[0] for r in rows}
    # all five variants of the element-wise kernels, three fence variants + modulo of the rest
    for v in range(5):
        assert f"k_stream<{v}, 1>" in names and f"k_gather32<{v}, 1>" in names and f"k_sum_partial<{v}>" in names
    for v in range(4):
        assert f"k_gemm_ring<{v}>" in names and f"k_rmsnorm_bf16<{v}>" in names
    fenced = [r for r in rows if r[1] in (1, 2) and (r[2] + r[3]) > 0]
    assert fenced and all(r[4] > 0 for r in fenced if r[1] == 1)        # the 32-bit fence shows up as v_and_b32
    # the fence costs at most a handful of registers (the paper: up to two at -O3)
    base = {r[0].replace("<1", "<0", 1): r for r in rows if r[1] == 0}
    for r in rows:
        if r[1] == 1 and r[0].replace("<1", "<0", 1) in base and "gemm" not in r[0]:
            assert r[5] - base[r[0].replace("<1", "<0", 1)][5] <= 4, r
