"""The assembly of the dense-layer kernels, checked on the CPU: no instruction touches a register that an
assembly-issued LDS read is still filling (see tests/asm_hazards.py).  Compiles paper_2503_01281_amd/csrc/dci_sage.hip to
assembly with the library's own flags (about 15 s)."""
import os
import subprocess

import pytest

from tests import asm_hazards

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_scanner_sees_a_planted_copy_and_accepts_a_waited_one():
    bad = """
_Zk:
	;;#ASMSTART
	ds_read_b128 v[4:7], v40 offset:0
	;;#ASMEND
	s_cbranch_vccz .LBB0_2
	v_mov_b64_e32 v[10:11], v[6:7]
	s_waitcnt lgkmcnt(0)
	v_mov_b64_e32 v[12:13], v[4:5]
"""
    hits = asm_hazards.scan(bad)
    assert [(h[0], h[2]) for h in hits] == [("_Zk", "v_mov_b64_e32 v[10:11], v[6:7]")]
    good = bad.replace("	v_mov_b64_e32 v[10:11], v[6:7]\n", "")
    assert asm_hazards.scan(good) == []
    # a read whose address register is still being filled, and one in another block after an unconditional branch
    chained = """
_Zk:
	;;#ASMSTART
	ds_read_b32 v3, v40
	ds_read_b32 v5, v3
	;;#ASMEND
	s_branch .LBB0_9
.LBB0_4:
	v_add_u32_e32 v5, 1, v5
"""
    hits = asm_hazards.scan(chained)
    assert len(hits) == 1 and hits[0][2] == "ds_read_b32 v5, v3"


def test_no_instruction_touches_a_fragment_register_before_its_wait(tmp_path):
    from paper_2503_01281_amd import build
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc here")
    out = tmp_path / "dci_sage.s"
    cmd = [hipcc] + [f for f in build.FLAGS if f != "-fPIC"] + ["-S", "--cuda-device-only", "-x", "hip",
                                                                 os.path.join(build.CSRC, "dci_sage.hip"), "-o", str(out)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    text = out.read_text()
    assert text.count(";;#ASMSTART") > 100          # the kernels' reads are there to be checked
    hits = asm_hazards.scan(text)
    assert hits == [], "\n".join(f"{k}:{ln}: {ins}   (read issued at line {rd})" for k, ln, ins, rd in hits[:20])
