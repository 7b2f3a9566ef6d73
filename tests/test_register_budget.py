"""The 256x256 bf16 product kernels must leave room for the weight-update kernel on the same compute unit.

Two wavefronts of a product workgroup share a SIMD's 512 registers per lane with the update kernel's wavefronts, which
need 64: above 224 registers per lane (or with spills) the update no longer runs beside the products and a training step
of the large configurations gets ~10 % slower without any test of the arithmetic noticing.  This compiles the device
code of csrc/gemm.hip with the library's own flags and reads the register counts out of the code object's metadata.
"""
import os
import re
import subprocess
import tempfile

import pytest

from paper_2403_11204_amd import build

SRC = os.path.join(build.CSRC, "gemm.hip")


@pytest.fixture(scope="module")
def kernel_metadata():
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "gemm.s")
        cmd = [build.hipcc()] + [a for a in build.COMMON if a != "-fPIC"] + ["--cuda-device-only", "-S", SRC, "-o", out]
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert r.returncode == 0, r.stdout[-2000:]
        text = open(out).read()
    meta = text[text.index("amdhsa.kernels"):]
    kernels = {}
    for entry in meta.split("- .agpr_count")[1:]:
        name = re.search(r"\.name:\s+(\S+)", entry).group(1)
        kernels[name] = {k: int(re.search(r"\.%s:\s+(\d+)" % k, entry).group(1))
                         for k in ("vgpr_count", "vgpr_spill_count", "private_segment_fixed_size")}
    return kernels


def test_big_product_kernels_fit_beside_the_update_kernel(kernel_metadata):
    big = {n: v for n, v in kernel_metadata.items() if "gemm_nt_big_kernel" in n}
    assert len(big) == 4, sorted(big)          # forward, data gradient, weight gradient, weight gradient + update
    for name, v in big.items():
        assert v["vgpr_count"] <= 224, (name, v)
        assert v["vgpr_spill_count"] == 0 and v["private_segment_fixed_size"] == 0, (name, v)


def test_no_product_kernel_spills(kernel_metadata):
    for name, v in kernel_metadata.items():
        if "gemm_nt" in name:
            assert v["vgpr_spill_count"] == 0, (name, v)
