"""Static check of the wavefront-per-model kernel's generated code (no GPU needed).

Every wavefront of that kernel pops its next model from the work queue with all 64 lanes taking part.
A pop under `if (lane == 0)` compiled into a kernel that never ended: the loop body finishes with
another branch on the same condition, the compiler joined the two across the back edge, and lanes
1..63 went round the loop on their own, past the pop.  In the generated code that shows as one more
loop level around the per-model body.  This test compiles two variants of the kernel to assembly and
checks that the loop nest is as deep as the source's (queue, epoch, step, chunk, inner loop) and no
deeper."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2012_04201_amd", "csrc")


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not on PATH")
def test_linear_kernel_loop_nest_is_the_sources(tmp_path):
    src = tmp_path / "probe.hip"
    src.write_text('#include "%s"\nnamespace {\n'
                   "template __global__ void k_train_linear<2, 1>(const TrainParams);\n"
                   "template __global__ void k_train_linear<16, 1>(const TrainParams);\n}\n"
                   % os.path.join(CSRC, "train_linear_f32.h"))
    out = tmp_path / "probe.s"
    cmd = ["hipcc", "-O3", "--offload-arch=gfx950", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "--cuda-device-only", "-S", str(src), "-o", str(out)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = out.read_text().split("\n")
    starts = [i for i, l in enumerate(lines) if "k_train_linear" in l and l.startswith("_Z") and ":" in l]
    assert len(starts) == 2
    for s in starts:
        e = next(i for i in range(s, len(lines)) if lines[i].startswith(".Lfunc_end"))
        depth = [int(m.group(1)) for l in lines[s:e] for m in [re.search(r"Loop Header: Depth=(\d+)", l)] if m]
        assert depth, "no loops found: the listing's annotations changed"
        # queue loop 1, epoch 2, step 3, chunk 4, the chunk's inner loops 5
        assert max(depth) == 5, depth
        body = "\n".join(lines[s:e])
        assert "global_atomic_add" in body and "s_endpgm" in body
