"""No kernel of the library may spill registers to scratch memory: the streaming GEMMs sit right at their
register budget (two workgroups per CU at 128 VGPRs), and a spill costs tens of percent without failing any
parity test.  Compiles the device code to assembly (no GPU needed) and reads every kernel's descriptor."""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("src", ["pv_kernels_matrix.hip", "pv_kernels_attention.hip", "pv_kernels_common.hip", "pv_kernels_vector.hip"])
def test_kernels_use_no_scratch(tmp_path, src):
    from paper_2505_01572_amd import build
    out = str(tmp_path / "k.s")
    flags = [f for f in build.FLAGS if f not in ("-fPIC", "-Wall", "-Wno-unused-function")]
    subprocess.run(["hipcc", *flags, "-S", "--offload-device-only", "-o", out, os.path.join(build.CSRC, src)],
                   check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    text = open(out).read()
    kernels = re.findall(r"\.amdhsa_kernel (\S+)(.*?)\.end_amdhsa_kernel", text, re.S)
    assert kernels, "no kernel descriptors found"
    spilled = [name for name, body in kernels if int(re.search(r"\.amdhsa_private_segment_fixed_size\s+(\d+)", body).group(1)) > 0]
    assert not spilled, f"kernels with scratch (register spills): {spilled}"
