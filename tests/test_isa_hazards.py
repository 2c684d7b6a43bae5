"""The inline-assembly DPP fmac of the real-input VALU kernel gets no automatic wait states.

A DPP instruction must not read a VGPR that a VALU instruction wrote in the two instructions before it, and must
not follow a write of EXEC within five.  The assembler inserts those waits for compiler-generated code only, so
this test compiles the device code to assembly and checks every `v_fmac_f32_dpp` in it.
"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _written_vgprs(ins: str):
    m = re.match(r"v_\w+\s+(?:v\[(\d+):(\d+)\]|v(\d+))", ins)
    if not m:
        return set()
    if m.group(1):
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    return {int(m.group(3))}


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not found")
def test_dpp_fmac_sources_are_not_fresh_valu_results(tmp_path):
    out = tmp_path / "api.s"
    cmd = ["hipcc", "-O3", "--offload-arch=gfx950", "-std=c++17", "-ffp-contract=off", "-Xclang", "-target-feature",
           "-Xclang", "-packed-fp32-ops", "-S", "--cuda-device-only", "-I", os.path.join(ROOT, "include"), "-o", str(out),
           os.path.join(ROOT, "paper_1706_09453_amd", "csrc", "bnn_api.hip")]
    subprocess.run(cmd, check=True, capture_output=True)
    code = [l.strip() for l in out.read_text().splitlines()]
    code = [l for l in code if l and not l.startswith((";", ".", "//")) and not l.endswith(":")]
    n_dpp, bad = 0, []
    for i, ins in enumerate(code):
        if not ins.startswith("v_fmac_f32_dpp"):
            continue
        n_dpp += 1
        src = int(re.match(r"v_fmac_f32_dpp v\d+, v(\d+),", ins).group(1))
        states, back = 0, 1          # wait states between the instruction `back` places earlier and this one
        while states < 5:
            prev = code[i - back]
            if states < 2 and prev.startswith("v_") and src in _written_vgprs(prev):
                bad.append((prev, ins))
            dst = prev.split(",")[0]
            if re.search(r"\bexec", dst) and (prev.startswith("s_") or prev.startswith("v_cmpx")):
                bad.append((prev, ins))
            m = re.match(r"s_nop\s+(\d+)", prev)
            states += int(m.group(1)) + 1 if m else 1
            back += 1
    assert n_dpp > 0, "the kernel no longer uses the DPP fmac: delete this test"
    assert not bad, bad[:5]
