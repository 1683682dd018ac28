"""The pass-2 kernel scales its logits with a hand-written v_fma_f32 that the compiler does not
analyse: it inserts no wait states between an MFMA and such a statement reading the MFMA's result.
The kernel therefore uses the statement only on accumulators written a whole sub-tile earlier.
This test compiles the kernels to ISA and checks that property on the listing: for every
hand-written v_fma_f32, the last MFMA (in listing order, within the kernel) that wrote its first
source register lies far more than the 18 wait states the slowest MFMA needs."""
import os
import re
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
MIN_DISTANCE = 32


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not installed")
def test_hand_written_fma_reads_only_settled_accumulators():
    src = os.path.join(ROOT, "paper_2503_12491_amd", "csrc", "window_scores.hip")
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "ws.s")
        subprocess.run(["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-I", os.path.join(ROOT, "include"),
                        "-I", os.path.dirname(src), "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                        "-S", "--cuda-device-only", "-o", out, src], check=True, capture_output=True)
        text = open(out).read()
    checked = 0
    for kern in re.split(r"\n(?=_ZN4cake\S+:)", text):
        name = kern.split(":")[0]
        if "scores_pass" not in name:
            continue
        idx, last, in_asm = 0, {}, False
        for line in kern.split("\n"):
            t = line.strip()
            if "ASMSTART" in t:
                in_asm = True
                continue
            if "ASMEND" in t:
                in_asm = False
                continue
            if not t or t[0] in ";." or t.endswith(":"):
                continue
            if t.startswith("s_endpgm"):
                break
            idx += 1
            m = re.match(r"v_mfma\S+ v\[(\d+):(\d+)\]", t)
            if m:
                for r in range(int(m.group(1)), int(m.group(2)) + 1):
                    last[r] = idx
            elif in_asm and t.startswith("v_fma_f32"):
                checked += 1
                src0 = int(re.findall(r"v(\d+)", t)[1])
                assert src0 not in last or idx - last[src0] >= MIN_DISTANCE, (name, t, idx - last[src0])
    assert checked > 0            # the statement is still in use; otherwise this test can go
