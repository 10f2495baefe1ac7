"""Checks on the generated gfx950 code of the kernels (no GPU needed: hipcc cross-compiles).

Two kernels name their direct-to-LDS loads as instructions with the base address in a scalar
register pair (`dma16s` in csrc/dlf_kernels.hip).  If the compiler ever ran out of scalar registers
there, it would substitute a vector register pair into the instruction text, which the assembler
accepts as a different, wrong addressing form; and a kernel that spills to scratch memory in its
multiply loops has lost the register budget it was written for.  Both show in the assembly."""
import os
import re
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2011_05630_amd", "csrc")


@pytest.fixture(scope="module")
def kernel_asm():
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "k.s")
        cmd = ["hipcc", "-O3", "-std=c++17", "--offload-arch=gfx950", "-x", "hip", "-S", "--cuda-device-only",
               "-I", os.path.join(ROOT, "include"), "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wno-unused-command-line-argument", "-o", out, os.path.join(CSRC, "dlf_kernels.hip")]
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert r.returncode == 0, r.stdout
        with open(out) as f:
            return f.read()


def _kernels(asm):
    """{mangled kernel name: body text} for every kernel entry point of the module."""
    names = re.findall(r"^\s*\.amdhsa_kernel\s+(\S+)", asm, flags=re.M)
    out = {}
    for n in names:
        # the whole function: a kernel with early exits has more than one s_endpgm
        m = re.search(r"^%s:.*?^\.Lfunc_end\d+:" % re.escape(n), asm, flags=re.M | re.S)
        assert m is not None, n
        out[n] = m.group(0)
    return out


def test_scalar_base_loads_name_scalar_registers(kernel_asm):
    ks = _kernels(kernel_asm)
    assert any("k_pwb" in n for n in ks) and any("k_c3b" in n for n in ks)
    seen = 0
    for name, body in ks.items():
        for line in body.splitlines():
            if "global_load_lds_dwordx4" not in line:
                continue
            ops = line.split("global_load_lds_dwordx4", 1)[1].strip()
            # either "v[a:b], off" (64-bit vector address) or "vN, s[a:b]" (scalar base + 32-bit offset)
            assert re.match(r"^(v\[\d+:\d+\], off|v\d+, s\[\d+:\d+\])(\s|$)", ops), (name, line.strip())
            seen += ops.startswith("v") and ", s[" in ops
    assert seen > 0, "the scalar-base form is expected in the block kernels"


def test_no_kernel_spills_to_scratch(kernel_asm):
    sizes = re.findall(r"^\s*\.amdhsa_kernel\s+(\S+).*?\.amdhsa_private_segment_fixed_size\s+(\d+)", kernel_asm,
                       flags=re.M | re.S)
    assert sizes
    for name, size in sizes:
        assert int(size) == 0, "%s uses %s bytes of scratch memory per lane" % (name, size)


def test_quantised_kernels_multiply_on_the_int8_matrix_instruction(kernel_asm):
    """The quantised forms of the block, pointwise-block and small-map kernels issue
    v_mfma_i32_32x32x32_i8 and no fp16 matrix instruction; their fp16 twins the reverse."""
    ks = _kernels(kernel_asm)
    quant = [n for n in ks if re.search(r"k_c3bILi\d+ELi\d+ELi\d+ELb1E|k_pwbILi\d+ELi\d+ELb0ELb1E|k_c3sILi\d+ELi\d+ELi\d+ELb1E", n)]
    assert len(quant) == 5 + 2 + 4, quant
    for n in quant:
        assert "v_mfma_i32_32x32x32_i8" in ks[n] and "v_mfma_f32_32x32x16_f16" not in ks[n], n
    twins = [n for n in ks if re.search(r"k_c3bILi\d+ELi\d+ELi\d+ELb0E|k_pwbILi\d+ELi\d+ELb\dELb0E|k_c3sILi\d+ELi\d+ELi\d+ELb0E", n)]
    assert len(twins) == 5 + 4 + 6, twins
    for n in twins:
        assert "v_mfma_f32_32x32x16_f16" in ks[n] and "v_mfma_i32" not in ks[n], n
