"""The row sort runs at the register limit of a 1024-thread workgroup (128 VGPRs): a small change can push the
compiler over it, and the kernel then spills into scratch memory and runs several times slower without any test
failing.  This test compiles the clustering kernels for gfx950 (no GPU needed) and reads the compiler's
resource remarks."""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def resource_remarks(source):
    from paper_2412_04180_amd import _build

    src = os.path.join(_build.CSRC, source)
    flags = [f for f in _build.HIPCC_FLAGS if f != "-shared"]
    cmd = [HIPCC] + flags + ["--cuda-device-only", "-c", "-Rpass-analysis=kernel-resource-usage", "-I",
                             os.path.join(ROOT, "include"), "-I", _build.CSRC, "-x", "hip", src, "-o", os.devnull]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout[-2000:]
    return r


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not installed")
def test_sort_kernel_variants_for_rows_up_to_12288_keep_their_keys_in_registers():
    r = resource_remarks("skim_cluster.hip")
    found = 0
    for variant in ("sort_kernelILi8ELb1E", "sort_kernelILi12ELb1E"):
        m = re.search(r"Function Name: \S*" + variant + r".*?LDS Size", r.stdout, re.S)
        assert m, f"no resource remarks for {variant}"
        scratch = int(re.search(r"ScratchSize \[bytes/lane\]: (\d+)", m.group(0)).group(1))
        vgprs = int(re.search(r"VGPRs: (\d+)", m.group(0)).group(1))
        assert scratch == 0, f"{variant} spills {scratch} bytes per lane into scratch memory"
        assert vgprs <= 128
        found += 1
    assert found == 2


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not installed")
def test_hessian_kernel_for_wide_layers_does_not_spill():
    """Two wavefronts per SIMD, 128 accumulator registers each: a reload from scratch memory inside the MFMA loop
    waits behind every tile load in flight (the memory counter is in-order)."""
    r = resource_remarks("skim_hessian.hip")
    m = re.search(r"Function Name: \S*xtx_big_kernel.*?LDS Size", r.stdout, re.S)
    assert m, "no resource remarks for xtx_big_kernel"
    scratch = int(re.search(r"ScratchSize \[bytes/lane\]: (\d+)", m.group(0)).group(1))
    occupancy = int(re.search(r"Occupancy \[waves/SIMD\]: (\d+)", m.group(0)).group(1))
    assert scratch == 0, f"xtx_big_kernel spills {scratch} bytes per lane into scratch memory"
    assert occupancy == 2
