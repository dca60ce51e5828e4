"""Register budget of the compiled convolution kernels (host-side check, no GPU).

The LDS-patch kernel keeps 4..16 accumulator tiles, a weight ring and the patch
prefetch in registers at two or three waves per SIMD.  A change that pushes a
variant over its budget does not fail any numerical test -- the compiler spills
to scratch memory and the layer just gets several times slower -- so the spill
counts the compiler reports are pinned here.
"""
import os
import re
import subprocess
import tempfile

import pytest

from paper_1908_05033_amd import build as B

CSRC = os.path.join(os.path.dirname(B.__file__), "csrc")
MAX_SPILLED_VGPRS = 40            # whole kernel
MAX_SCRATCH_IN_MFMA_BLOCK = 48    # scratch instructions in a basic block that issues MFMAs


def _device_asm(src):
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "k.s")
        flags = [f for f in B.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
        cmd = [os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")] + flags + ["-S", "--cuda-device-only", "-o", out, src]
        proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert proc.returncode == 0, proc.stdout[-2000:]
        return open(out).read()


@pytest.mark.parametrize("source", ["conv_patch_c4r3.hip", "conv_patch_c4r1.hip", "conv_patch_c2r3.hip", "conv_patch_c2r1.hip",
                                    "conv_patch_c3r3.hip", "conv_patch_c3r1.hip",
                                    "conv_simple.hip", "conv_fc.hip", "quantize_act.hip"])
def test_kernels_stay_inside_their_register_budget(source):
    asm = _device_asm(os.path.join(CSRC, source))
    kernels = re.findall(r"\.name:\s+(\S+).*?\.vgpr_count:\s+(\d+).*?\.vgpr_spill_count:\s+(\d+)", asm, re.S)
    assert kernels, "no kernel metadata found in the device assembly"
    over = [(n, int(v), int(s)) for n, v, s in kernels if int(s) > MAX_SPILLED_VGPRS]
    assert not over, "kernels spilling more than %d registers: %s" % (MAX_SPILLED_VGPRS, over[:5])
    # no variant may spill inside the blocks that feed the matrix cores
    hot = []
    for fn in re.split(r"\n(?=_Z\S+:)", asm):
        name = fn.split(":", 1)[0]
        for block in re.split(r"\n\.LBB\d+_\d+:", fn):
            ins = [l.split()[0] for l in block.splitlines() if l.startswith("\t") and not l.startswith("\t.")]
            if sum("mfma" in i for i in ins) >= 8:
                n_scratch = sum(i.startswith("scratch_") for i in ins)
                if n_scratch > MAX_SCRATCH_IN_MFMA_BLOCK:
                    hot.append((name, n_scratch))
    assert not hot, "scratch traffic inside MFMA blocks: %s" % hot[:5]
