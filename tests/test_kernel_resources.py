"""Host-side guard on what the compiler made of the attention kernels: none of them may keep
values in scratch memory (a handful of registers spilled inside the tile loop cost 4-8 % at D = 64,
and which values spill changes with any edit), and each must reach the occupancy its launch
geometry assumes.  Compiles the source once with resource-usage remarks; no GPU needed."""
import os
import re
import subprocess

import pytest

from paper_2509_22323_amd import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def usage(tmp_path_factory):
    out = tmp_path_factory.mktemp("res") / "x.so"
    cmd = [build.HIPCC] + build.FLAGS + ["-Rpass-analysis=kernel-resource-usage", "-o", str(out)] + build.SOURCES
    err = subprocess.run(cmd, capture_output=True, text=True, check=True).stderr
    kernels, cur = {"__stderr__": err}, None
    for line in err.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            cur = kernels.setdefault(m.group(1), {})
        for key in ("VGPRs", "ScratchSize [bytes/lane]", "Occupancy [waves/SIMD]", "LDS Size [bytes/block]"):
            m = re.search(re.escape(key) + r": (\d+)", line)
            if m and cur is not None and key not in cur:
                cur[key] = int(m.group(1))
    return kernels


WANT = {  # kernel name fragment -> waves per SIMD its launch plan counts on
    "attn_dense_pp_kernelILi64E": 4, "attn_dense_pp_kernelILi128E": 2,
    "attn_sparse_sg_kernelILi64E": 4, "attn_sparse_sg_kernelILi128E": 2,
    "attn_sparse_pp_kernelILi64ELi2E": 2, "attn_sparse_pp_kernelILi128ELi2E": 1,
}


@pytest.mark.parametrize("fragment,occupancy", sorted(WANT.items()))
def test_attention_kernels_stay_in_registers(usage, fragment, occupancy):
    name = [k for k in usage if fragment in k]
    assert len(name) == 1, (fragment, list(usage))
    u = usage[name[0]]
    assert u["ScratchSize [bytes/lane]"] == 0, u
    assert u["Occupancy [waves/SIMD]"] >= occupancy, u


def test_no_kernel_of_the_library_uses_scratch_memory(usage):
    """(Attention, planners, selection and Cache-Reuse kernels alike: a value that is spilled inside a
    divergent region comes back stale for the lanes that sat the region out.)"""
    kernels = {k: u for k, u in usage.items() if k != "__stderr__"}
    assert len(kernels) >= 20, sorted(kernels)
    bad = {k: u for k, u in kernels.items() if u.get("ScratchSize [bytes/lane]", 0) != 0}
    assert not bad, bad


def test_the_library_compiles_without_warnings(usage):
    """(-Wall is on; the host pass's note about the packed-fp32 target feature is not a warning of the code.)"""
    bad = [l for l in usage["__stderr__"].splitlines() if "warning:" in l and "packed-fp32-ops" not in l]
    assert not bad, bad
