"""Static check of the kernels' assembly: no MFMA result is read before its wait states have passed, on any
control-flow path (paper_2502_06766_amd/isa_check.py says why this is checked)."""
import os
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_2502_06766_amd import build as hip_build
from paper_2502_06766_amd import isa_check

MFMA_SOURCES = ["scan.hip", "tail.hip", "pages.hip", "index8.hip"]     # the sources whose kernels use MFMA


def _assembly(src, out_dir):
    out = os.path.join(out_dir, src.replace(".hip", ".s"))
    subprocess.check_call([hip_build.HIPCC, *hip_build.FLAGS, '-DTKA_BUILD_ID="isa"', "-S", "--offload-device-only",
                           os.path.join(hip_build.CSRC, src), "-o", out], stderr=subprocess.DEVNULL)
    return out


def test_no_mfma_result_is_read_early():
    with tempfile.TemporaryDirectory() as d:
        with ThreadPoolExecutor(max_workers=4) as ex:
            files = list(ex.map(lambda s: _assembly(s, d), MFMA_SOURCES))
        total = 0
        for f in files:
            text = open(f).read()
            total += text.count("v_mfma")
            hits = isa_check.check(f)
            assert not hits, f"{os.path.basename(f)}: " + "; ".join(f"{h[0][:50]} line {h[1]}: read after {h[2]} wait states ({h[4]})" for h in hits[:5])
        assert total > 1000          # the check saw the kernels (thousands of MFMAs over all instantiations)


def test_the_check_finds_a_planted_early_read():
    lines = """_Zkernel:
	v_mfma_f32_16x16x32_f16 a[0:3], v[2:5], v[10:13], 0
	s_cbranch_scc1 .LBB0_2
	s_nop 7
	v_accvgpr_read_b32 v1, a1
.LBB0_2:
	v_accvgpr_read_b32 v0, a0
	s_endpgm
.Lfunc_end0:
""".splitlines()
    hits = isa_check._check_lines(lines, 8)
    assert len(hits) == 1 and hits[0][2] == 1 and "a0" in hits[0][4]
