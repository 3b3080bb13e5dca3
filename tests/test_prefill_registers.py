"""The prefill kernel names its 256 accumulation registers outright in inline asm and tells the compiler only
that they are written.  That is sound as long as the compiler itself never touches an accumulation register
and spills nothing: this test compiles the file to gfx950 assembly (no GPU needed) and checks exactly that,
for every instantiation of the kernel."""
import os
import re
import subprocess

import pytest

from paper_2410_13461_amd import build as pmpd_build

SRC = os.path.join(pmpd_build.CSRC, "pmpd_prefill.hip")


@pytest.fixture(scope="module")
def assembly(tmp_path_factory):
    out = tmp_path_factory.mktemp("prefill_asm") / "pmpd_prefill.s"
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in pmpd_build.HIPCC_FLAGS if f not in ("-fPIC", "-shared")]
    cmd = [hipcc, *flags, "-I" + os.path.join(pmpd_build.ROOT, "include"), "-I" + pmpd_build.CSRC, "-S", "--cuda-device-only",
           "-o", str(out), SRC]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout
    return out.read_text().split("\n")


def _kernels(lines):
    """(name, body lines) of every prefill kernel in the assembly."""
    out = []
    for i, line in enumerate(lines):
        m = re.match(r"^(_ZN4pmpd\w*prefill\w*):", line)
        if m:
            end = next(j for j in range(i, len(lines)) if "s_endpgm" in lines[j])
            out.append((m.group(1), lines[i:end + 1]))
    return out


def test_compiler_never_touches_an_accumulation_register(assembly):
    kernels = _kernels(assembly)
    assert len(kernels) == 6  # layer and stack kernel at b = 4, 3, 2
    for name, body in kernels:
        in_asm = False
        mfma = 0
        for line in body:
            if "ASMSTART" in line:
                in_asm = True
                continue
            if "ASMEND" in line:
                in_asm = False
                continue
            code = line.split(";")[0]
            if in_asm:
                mfma += "v_mfma_f32_16x16x32_f16" in code
                continue
            assert not re.search(r"\ba\[?\d|accvgpr", code), f"{name}: compiler-made use of an accumulation register: {line.strip()}"
        # the group body is written out for both parities: 2 x 4 K-steps x 64
        assert mfma == 512, (name, mfma)


def test_no_spills_and_all_accumulators_counted(assembly):
    text = "\n".join(assembly)
    blocks = re.findall(r"\.agpr_count:\s+(\d+).*?\.name:\s+(\S+).*?\.vgpr_count:\s+(\d+)\s+\.vgpr_spill_count:\s+(\d+)", text, flags=re.S)
    seen = 0
    for agpr, name, vgpr, spill in blocks:
        if "prefill" not in name:
            continue
        seen += 1
        assert int(agpr) == 256, (name, agpr)
        assert int(spill) == 0, (name, spill)
        assert int(vgpr) <= 512, (name, vgpr)
    assert seen == 6
