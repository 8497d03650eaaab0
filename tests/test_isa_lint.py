"""The kernels that issue loads by hand must never have those registers copied or spilled while the
data is on its way (the compiler cannot see that it is), and no kernel may read a matrix-core result
behind a basic-block boundary before the product has been delivered.  Compiles the sources to ISA
text and runs the lints over every kernel in them."""
import os
import shutil
import subprocess

import pytest

from tests import isa_lint

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


@pytest.mark.parametrize("source", ["kernels_gemm.hip", "kernels_layers.hip"])
def test_no_compiler_access_to_registers_of_loads_in_flight(source, tmp_path):
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not available")
    out = tmp_path / (source + ".s")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-S", "--cuda-device-only", "-o", str(out),
           os.path.join(ROOT, "paper_2605_13319_amd", "csrc", source)]
    subprocess.run(cmd, check=True, capture_output=True)
    text = out.read_text()
    assert "global_load_dwordx4" in text and "ASMSTART" in text  # the listing holds what the lint looks for
    assert isa_lint.check(str(out)) == 0


@pytest.mark.parametrize("source", ["kernels_gemm.hip", "kernels_layers.hip", "kernels_attn.hip", "kernels_gemm_wide.hip"])
def test_no_early_read_of_matrix_core_results_across_blocks(source, tmp_path):
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not available")
    out = tmp_path / (source + ".s")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-S", "--cuda-device-only", "-o", str(out),
           os.path.join(ROOT, "paper_2605_13319_amd", "csrc", source)]
    subprocess.run(cmd, check=True, capture_output=True)
    assert "v_mfma" in out.read_text()
    assert isa_lint.check_mfma(str(out)) == 0


def test_lint_flags_an_early_read_of_a_matrix_core_result(tmp_path):
    """An LDS store of an accumulator right behind a branch target is flagged; with the padding
    spelled out in front of the branch it is not; a store in the v_mfma's own block is the compiler's
    business and is not looked at."""
    bad = """
kern:
	s_cbranch_scc1 .LBB0_2
	v_mfma_f32_16x16x32_bf16 v[4:7], v[8:11], v[12:15], v[4:7]
.LBB0_2:
	s_or_b64 exec, exec, s[2:3]
	ds_write_b128 v1, v[4:7]
	s_endpgm
"""
    good = bad.replace(".LBB0_2:", "\ts_nop 15\n\ts_nop 7\n.LBB0_2:")
    same_block = bad.replace(".LBB0_2:\n\ts_or_b64 exec, exec, s[2:3]\n", "")
    for name, text, want in (("bad", bad, 1), ("good", good, 0), ("same", same_block, 0)):
        p = tmp_path / (name + ".s")
        p.write_text(text)
        assert isa_lint.check_mfma(str(p)) == want, name


def test_lint_flags_a_copy_before_the_wait(tmp_path):
    """The lint itself: a listing in which the compiler copies a hand-loaded register before the
    hand-issued wait is flagged, the same listing with the copy after the wait is not."""
    bad = """
kern:
	;;#ASMSTART
	global_load_dwordx4 v[4:7], v[2:3], off nt
	;;#ASMEND
	s_cbranch_scc1 .LBB0_2
	v_mov_b32_e32 v9, v5
.LBB0_2:
	;;#ASMSTART
	s_waitcnt vmcnt(0)
	;;#ASMEND
	v_add_f32_e32 v1, v4, v9
	s_endpgm
"""
    good = bad.replace("\tv_mov_b32_e32 v9, v5\n", "").replace("\tv_add_f32_e32 v1, v4, v9\n",
                                                               "\tv_mov_b32_e32 v9, v5\n\tv_add_f32_e32 v1, v4, v9\n")
    pb, pg = tmp_path / "bad.s", tmp_path / "good.s"
    pb.write_text(bad)
    pg.write_text(good)
    assert isa_lint.check(str(pb)) == 1
    assert isa_lint.check(str(pg)) == 0
