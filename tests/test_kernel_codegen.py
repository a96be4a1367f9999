"""Guard of the tile kernel's generated code (CPU only: hipcc cross-compiles gfx950 to assembly).

The pipeline of ``match_tile_kernel`` rests on one hand-placed wait per step (``s_waitcnt vmcnt(8)``:
everything but the newest pool slice has landed).  The direct-to-LDS operand loads are inline
assembly, so the compiler does not count them: any wait on the memory counter that it adds inside a
step on its own (for a spilled register that it reloads there, for instance) waits for the operand
loads of the step as well and serialises the pipeline, silently: results stay right, the kernel
just gets slower.  Which registers are spilled where changes with every edit of the kernel, so the
assembly of every instantiation is checked: in the steady-state loops (the basic blocks that hold
the matrix instructions and fragment reads of a step) there is exactly the one wait on the memory
counter, and no access to scratch memory.
"""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2507_21433_amd", "csrc")


@pytest.fixture(scope="module")
def assembly(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("asm") / "rc_match.s")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-Wno-inline-asm", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-S",
           "--cuda-device-only", "-o", out, os.path.join(CSRC, "rc_match.hip")]
    subprocess.run(cmd, check=True, capture_output=True, text=True, timeout=600)
    return open(out).read()


def kernels(asm):
    """(name, body) of every match_tile_kernel instantiation."""
    for m in re.finditer(r"\n(_ZN2rc17match_tile_kernelI\w+):", asm):
        end = asm.index(".Lfunc_end", m.end())
        yield m.group(1), asm[m.end():end]


def test_every_instantiation_is_there(assembly):
    names = [n for n, _ in kernels(assembly)]
    # f16 and bf16 x (256x256 in modes 0-4, 256x64 and 256x128 in mode 0)
    assert len(names) == 16, names


def test_steady_state_loops_wait_once_and_never_touch_scratch(assembly):
    checked = 0
    for name, body in kernels(assembly):
        blocks = re.split(r"\n(\.LBB\d+_\d+):", body)
        loops = 0
        for label, text in zip(blocks[1::2], blocks[2::2]):
            back = re.search(r"s_cbranch_\w+ " + re.escape(label) + r"\n", text)
            if back:
                text = text[:back.end()]   # what follows the branch back to the loop head is the code after the loop
            if text.count("v_mfma") < 4 * 4 or text.count("ds_read_b128") < 16 or "s_barrier" not in text:
                continue   # not a pipeline step (phase ends, epilogue)
            loops += 1
            # (a wait for "at most 63 outstanding" is the counter's maximum, i.e. no wait at all)
            waits = [l.strip() for l in text.split("\n") if "s_waitcnt" in l and "vmcnt" in l and "vmcnt(63)" not in l]
            assert waits == ["s_waitcnt vmcnt(8)"], (name, label, waits)
            assert "scratch_" not in text, (name, label, [l.strip() for l in text.split("\n") if "scratch_" in l])
            assert text.count("buffer_load_dwordx4") >= 10, (name, label)   # the step's refills ride between the matrix instructions
            checked += 1
        assert loops >= 1, f"no steady-state loop recognised in {name}"
    assert checked >= 16
