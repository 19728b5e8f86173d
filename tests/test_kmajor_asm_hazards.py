"""The K-major GEMM path reads its LDS fragments from inline assembly with hand-placed waits.  The source ties each
result to the wait that covers it; this test compiles the kernel file to gfx950 assembly (no GPU needed) and checks the
generated code itself: no instruction touches the destination of an LDS read that no `s_waitcnt lgkmcnt` has retired
yet, on any path through any of the kernels.  Planted mistakes show that the checker sees one when it is there."""
import os
import re
import subprocess

import pytest

from tests import asm_lds_hazards as hz
from paper_2502_16982_amd import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

GOOD = """
kern:
	ds_read_b64_tr_b16 v[4:5], v1
	ds_read_b64_tr_b16 v[6:7], v1 offset:1024
	ds_read_b128 v[8:11], v2
	s_waitcnt lgkmcnt(1)
	v_mfma_f32_32x32x16_bf16 v[16:31], v[4:7], v[12:15], v[16:31]
	s_waitcnt lgkmcnt(0)
	v_mfma_f32_32x32x16_bf16 v[16:31], v[4:7], v[8:11], v[16:31]
	s_endpgm
.Lfunc_end0:
"""


def test_checker_accepts_correct_code_and_flags_planted_mistakes():
    assert hz.check_file_text(GOOD) == {"kern": []}
    # a wait that leaves one read too many outstanding
    bad = GOOD.replace("s_waitcnt lgkmcnt(1)", "s_waitcnt lgkmcnt(2)")
    v = hz.check_file_text(bad)["kern"]
    assert len(v) == 1 and "v[6, 7]" in v[0]
    # a copy of a result before it has landed
    bad = GOOD.replace("	ds_read_b128 v[8:11], v2\n", "	ds_read_b128 v[8:11], v2\n	v_mov_b32_e32 v40, v5\n")
    assert len(hz.check_file_text(bad)["kern"]) == 1
    # reads issued at the end of a loop body and consumed at its top: the walk follows the back edge
    loop = """
kern:
	ds_read_b128 v[8:11], v2
.LBB0_1:
	v_mfma_f32_32x32x16_bf16 v[16:31], v[8:11], v[12:15], v[16:31]
	ds_read_b128 v[8:11], v2
	s_waitcnt lgkmcnt(0)
	s_cbranch_scc1 .LBB0_1
	s_endpgm
.Lfunc_end0:
"""
    v = hz.check_file_text(loop)["kern"]
    assert len(v) == 1 and "v_mfma" in v[0]          # first pass through the loop head: nothing waited yet
    assert hz.check_file_text(loop.replace(".LBB0_1:\n", "	s_waitcnt lgkmcnt(0)\n.LBB0_1:\n"))["kern"] == []
    # a scalar load in between shares the counter but cannot make an LDS read look finished
    with_smem = GOOD.replace("	ds_read_b128 v[8:11], v2\n", "	s_load_dwordx2 s[4:5], s[0:1], 0x0\n	ds_read_b128 v[8:11], v2\n")
    assert hz.check_file_text(with_smem) == {"kern": []}


@pytest.fixture(scope="module")
def gemm_asm(tmp_path_factory):
    out = tmp_path_factory.mktemp("asm") / "kernels_gemm_bf16.s"
    cmd = [build.hipcc_path(), *build.HIPCC_FLAGS, "-S", "--cuda-device-only",
           os.path.join(build.CSRC, "kernels_gemm_bf16.hip"), "-o", str(out)]
    proc = subprocess.run(cmd, capture_output=True, text=True, cwd=str(out.parent))
    assert proc.returncode == 0, proc.stderr[-2000:]
    return out.read_text()


def test_generated_gemm_code_waits_for_every_lds_read_it_uses(gemm_asm):
    kernels = hz.split_kernels(gemm_asm)
    gemm = {k: v for k, v in kernels.items() if "ns_gemm_bf16" in k}
    assert len(gemm) == 12                       # fine and coarse kernel x {k-contiguous, K-major} x {1, 2, 3} planes
    assert sum("ds_read_b64_tr_b16" in t for k in gemm for _, t in gemm[k]) >= 100   # the K-major reads are there
    for name, lines in gemm.items():
        assert hz.check_kernel(lines) == [], name


def test_a_loosened_wait_in_the_generated_code_is_caught(gemm_asm):
    """Sensitivity on the real thing: the first hand-placed wait after a transposing read, loosened by two."""
    lines = gemm_asm.splitlines()
    first_tr = next(i for i, l in enumerate(lines) if "ds_read_b64_tr_b16" in l)
    for i in range(first_tr, len(lines)):
        m = re.search(r"s_waitcnt lgkmcnt\((\d+)\)", lines[i])
        if m:
            lines[i] = lines[i].replace(m.group(0), "s_waitcnt lgkmcnt(%d)" % (int(m.group(1)) + 2))
            break
    res = hz.check_file_text("\n".join(lines))
    assert any(v for v in res.values())
