"""The device compile flags do what the build file says: with them, a kernel whose plain -O3 build contains
packed fp32 vector instructions contains none."""
import os
import re
import subprocess
import tempfile

import pytest

from paper_2511_10676_amd import build

PACKED = re.compile(r"\bv_pk_(add|mul|fma)_f32\b")


def _asm(flags):
    src = os.path.join(build.CSRC, "predict_simple.hip")
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "k.s")
        cmd = [build._hipcc(), *flags, "-x", "hip", "--cuda-device-only", "-S", src, "-o", out]
        subprocess.run(cmd, check=True, capture_output=True)
        return open(out).read()


def test_packed_fp32_instructions_are_switched_off_in_device_code():
    try:
        build._hipcc()
    except RuntimeError:
        pytest.skip("hipcc not installed")
    with_flags = _asm(build.HIPCC_FLAGS)
    assert not PACKED.search(with_flags), "packed fp32 instruction in a build with the library's flags"
    # the check bites: the same file without the feature switch does contain them
    bare = [f for f in build.HIPCC_FLAGS if f not in ("-Xclang", "-target-feature", "-packed-fp32-ops")]
    assert PACKED.search(_asm(bare)), "the witness kernel no longer contains packed fp32 instructions without the switch"
