"""Compile-time checks of the greedy-loop kernel (CPU only: hipcc cross-compiles for gfx950).

Resources: the kernel runs 1024 threads per workgroup, which leaves each thread 128 vector registers.  A change
that pushes it over that limit makes the compiler spill to scratch memory, and the kernel then runs some 40%
slower: a performance guard.

Ordering: the one place where the kernel's correctness rests on the ORDER in which a wavefront's LDS operations
are issued is the early publication of the next step's candidate: a column's wavefront merges its key into the
workgroup's minimum, counts itself, and reads the minimum back; the wavefront whose count comes out last
publishes what it read.  LDS executes one wavefront's operations in issue order, so the last counter's read sees
every other column's key (each was issued ahead of its own count) -- provided the three operations leave the
compiler in program order.  They are relaxed atomics on two addresses, which the language would let a compiler
reorder; the second test reads the generated code and fails if it ever does."""
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
    assert len(loops) == 5, "expected W in LDS / in the workspace, each for one layer and for several per launch, and the long-block form"
    for k in loops:
        name = k.split()[0]
        scratch = int(re.search(r"ScratchSize \[bytes/lane\]: (\d+)", k).group(1))
        vgprs = int(re.search(r"\bVGPRs: (\d+)", k).group(1))
        assert scratch == 0, "%s spills %d bytes per lane to scratch memory" % (name, scratch)
        assert vgprs <= 128, "%s needs %d vector registers" % (name, vgprs)


def test_candidate_merge_count_and_read_back_are_issued_in_program_order(tmp_path):
    """ds_min_u64 (key into the workgroup's minimum) -> ds_add_rtn_u32 (count) -> ds_read_b64 (minimum back, same
    address as the ds_min), back to back, once in each of the five instantiations."""
    from paper_2302_04089_amd import build
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    src = os.path.join(build.CSRC, "prune_lazy.hip")
    asm = tmp_path / "k.s"
    cmd = [hipcc] + build.FLAGS + build.FILE_FLAGS.get("prune_lazy.hip", []) + ["--cuda-device-only", "-S", src, "-o", str(asm)]
    out = subprocess.run(cmd, capture_output=True, text=True)
    assert out.returncode == 0, out.stderr[-2000:]
    insts = [l.split(";")[0].strip() for l in asm.read_text().splitlines()]
    insts = [l for l in insts if l and not l.startswith((".", "s_nop")) and not l.endswith(":")]
    counted = [i for i, l in enumerate(insts) if l.startswith("ds_add_rtn_u32")]
    assert len(counted) == 5, "one counting atomic per kernel instantiation expected, found %d" % len(counted)
    for i in counted:
        before, after = insts[i - 1], insts[i + 1]
        assert before.startswith("ds_min_u64"), "the count is not issued right behind the key merge: %r" % before
        assert after.startswith("ds_read_b64"), "the read-back is not issued right behind the count: %r" % after
        off_min = re.search(r"offset:(\d+)", before).group(1)
        off_read = re.search(r"offset:(\d+)", after).group(1)
        addr_min = before.split()[1].rstrip(",")
        addr_read = after.split()[2].rstrip(",")
        assert off_min == off_read and addr_min == addr_read, "read-back and merge address differ: %r / %r" % (before, after)
