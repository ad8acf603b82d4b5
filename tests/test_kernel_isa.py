"""Two properties of the kernels' ISA, checked on the assembly (no GPU needed; compiling the two kernel
files takes about a minute).

1. No scalar load with a register offset.  hipcc turned `kernel_argument.array[g]` (a by-value kernel
   argument indexed with a run-time value) into `s_load_dwordx2 dst, base, soffset` with a base advanced
   by g and an offset register of 7 g: only their sum is a multiple of four, the scalar memory unit drops
   the low bits of each, and the load returned halves of two neighbouring pointers (a memory fault on the
   GPU).  The sources now stage such structs in LDS.

2. No register spills on the paths every workgroup runs.  The layer launch lost a fifth of its time to
   scratch traffic while its piece loop spilled (16 MB of scratch writes per launch); what is left are a
   few registers around the front units of the select build."""
import functools
import os
import re
import subprocess
import tempfile

import pytest

from paper_2602_04541_amd import build as lbuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FORM = re.compile(r"^\s*s_(buffer_)?load_dword(x\d+)?\s+[^;]*\],\s*s\d+(\s|$)")
SOURCES = ["lychee_layer.hip", "lychee_units.hip"]


@functools.lru_cache(maxsize=None)
def assembly(source: str) -> str:
    flags = [f for f in lbuild.FLAGS if f not in ("-shared", "-fPIC")]
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, source + ".s")
        cmd = [lbuild.hipcc()] + flags + ["-S", "--cuda-device-only", "-I", os.path.join(ROOT, "include"),
                                          os.path.join(lbuild.CSRC, source), "-o", out]
        subprocess.check_call(cmd, stderr=subprocess.DEVNULL)
        text = open(out).read()
    assert "s_endpgm" in text, "no kernel in the assembly"
    return text


def scratch_bytes(text: str) -> dict:
    """Kernel name (mangled) -> bytes of scratch memory per lane, from the code object's metadata."""
    out = {}
    name = None
    size = None
    for line in text.splitlines():
        m = re.match(r"\s*\.private_segment_fixed_size:\s*(\d+)", line)
        if m:
            size = int(m.group(1))
        m = re.match(r"\s*\.name:\s*(\S+)", line)
        if m:
            name = m.group(1)
        if line.strip().startswith(".vgpr_spill_count") and name is not None and size is not None:
            out[name] = size
            name = size = None
    return out


@pytest.mark.parametrize("source", SOURCES)
def test_no_scalar_load_with_a_register_offset(source):
    hits = [line.strip() for line in assembly(source).splitlines() if FORM.match(line)]
    assert not hits, "scalar loads with a register offset: %s" % hits[:5]


def test_the_piece_paths_do_not_spill():
    layer = scratch_bytes(assembly("lychee_layer.hip"))
    units = scratch_bytes(assembly("lychee_units.hip"))
    assert layer and units
    dense = [v for k, v in layer.items() if "lychee_layer_kernelILb0ELi0" in k]
    hybrid = [v for k, v in layer.items() if "lychee_layer_kernelILb1ELi1" in k]
    assert dense == [0], layer
    assert len(hybrid) == 1 and hybrid[0] <= 64, layer      # a few registers around its front units
    pooled = {k: v for k, v in units.items() if "lychee_pool_kernel" in k}
    assert pooled and all(v == 0 for v in pooled.values()), pooled
