"""Host-side check of what the compiler made of the kernels: no kernel may use scratch memory
(register spills) and none may exceed the 160 KiB of LDS of a compute unit.

Spills are more than a speed matter here. The kernels order their direct-to-LDS copies by
counting outstanding vector-memory instructions (s_waitcnt vmcnt(n)); a spill store completes
out of order with respect to loads and would make such a count pass early, and a spill reload
makes the compiler wait for every copy in flight. The check compiles the two kernel files for
gfx950 with the flags of the build and reads the compiler's resource remarks (no GPU needed)."""
import concurrent.futures
import os
import re
import subprocess

import pytest

from paper_2307_08691_amd import build as fa_build


def resource_remarks(source):
    cmd = [fa_build.hipcc(), *[f for f in fa_build.FLAGS if f not in ("-shared", "-fPIC")], "--cuda-device-only", "-c",
           "-Rpass-analysis=kernel-resource-usage", "-o", os.devnull, os.path.join(fa_build.CSRC, source)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    kernels, cur = {}, None
    for line in r.stderr.splitlines():
        m = re.search(r"remark: (?:Function Name: (\S+)|\s*(ScratchSize \[bytes/lane\]|LDS Size \[bytes/block\]|VGPRs Spill|SGPRs Spill): (\d+))", line)
        if not m:
            continue
        if m.group(1):
            cur = kernels.setdefault(m.group(1), {})
        elif cur is not None:
            cur[m.group(2)] = int(m.group(3))
    return kernels


@pytest.fixture(scope="module")
def remarks():
    with concurrent.futures.ThreadPoolExecutor(2) as ex:
        a, b = ex.map(resource_remarks, ["fa_fwd.hip", "fa_bwd.hip"])
    return {**a, **b}


def test_every_kernel_was_seen(remarks):
    names = " ".join(remarks)
    for k in ("fwd_kernel", "fwd_merge_kernel", "bwd_prep_kernel", "bwd_dkdv_kernel", "bwd_dq_kernel"):
        assert k in names
    assert len(remarks) >= 60  # every instantiation reports


def test_no_kernel_spills_or_uses_scratch(remarks):
    bad = {k: v for k, v in remarks.items() if v.get("ScratchSize [bytes/lane]", 0) or v.get("VGPRs Spill", 0)}
    assert not bad, bad


def test_lds_fits_a_compute_unit(remarks):
    assert max(v.get("LDS Size [bytes/block]", 0) for v in remarks.values()) <= 160 * 1024
