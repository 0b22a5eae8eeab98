"""Compile-time resource check of the greedy-loop kernel (CPU only: hipcc cross-compiles for gfx950).

The kernel runs 1024 threads per workgroup, which leaves each thread 128 vector registers.  A change
that pushes it over that limit makes the compiler spill to scratch memory: the kernel then runs some
40% slower, and variants that spilled have also produced wrong removal orders on the GPU.  All
instantiations must therefore stay free of scratch memory."""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_greedy_loop_kernel_uses_no_scratch_memory(tmp_path):
    from paper_2302_04089_amd import build
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    src = os.path.join(build.CSRC, "prune_lazy.hip")
    cmd = [hipcc] + build.FLAGS + build.FILE_FLAGS.get("prune_lazy.hip", []) + [
        "--cuda-device-only", "-Rpass-analysis=kernel-resource-usage", "-c", src, "-o", str(tmp_path / "k.o")]
    out = subprocess.run(cmd, capture_output=True, text=True)
    assert out.returncode == 0, out.stderr[-2000:]
    kernels = re.split(r"remark: Function Name: ", out.stderr)[1:]
    loops = [k for k in kernels if "prune_lazy_kernel" in k.split()[0]]
    assert len(loops) == 4, "expected W in LDS / in the workspace, each for one layer and for several per launch"
    for k in loops:
        name = k.split()[0]
        scratch = int(re.search(r"ScratchSize \[bytes/lane\]: (\d+)", k).group(1))
        vgprs = int(re.search(r"\bVGPRs: (\d+)", k).group(1))
        assert scratch == 0, "%s spills %d bytes per lane to scratch memory" % (name, scratch)
        assert vgprs <= 128, "%s needs %d vector registers" % (name, vgprs)
