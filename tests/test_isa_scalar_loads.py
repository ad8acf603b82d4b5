"""The kernels' ISA must hold no scalar load with a register offset.

hipcc turned `kernel_argument.array[g]` (a by-value kernel argument indexed with a run-time value) into
`s_load_dwordx2 dst, base, soffset` with a base advanced by g and an offset register of 7 g: only
their sum is a multiple of four, the scalar memory unit drops the low bits of each, and the load
returned halves of two neighbouring pointers (a memory fault on the GPU).  The sources now stage
such structs in LDS; this test compiles the two kernel files to assembly (no GPU needed, about a
minute each) and fails if the form comes back."""
import os
import re
import subprocess
import tempfile

import pytest

from paper_2602_04541_amd import build as lbuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FORM = re.compile(r"^\s*s_(buffer_)?load_dword(x\d+)?\s+[^;]*\],\s*s\d+(\s|$)")


@pytest.mark.parametrize("source", ["lychee_layer.hip", "lychee_units.hip"])
def test_no_scalar_load_with_a_register_offset(source):
    flags = [f for f in lbuild.FLAGS if f not in ("-shared", "-fPIC")]
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, source + ".s")
        cmd = [lbuild.hipcc()] + flags + ["-S", "--cuda-device-only", "-I", os.path.join(ROOT, "include"),
                                          os.path.join(lbuild.CSRC, source), "-o", out]
        subprocess.check_call(cmd, stderr=subprocess.DEVNULL)
        text = open(out).read()
    assert "s_endpgm" in text, "no kernel in the assembly"
    hits = [line.strip() for line in text.splitlines() if FORM.match(line)]
    assert not hits, "scalar loads with a register offset: %s" % hits[:5]
