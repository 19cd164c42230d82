"""Host-side check of what the compiler made of the kernels: no kernel may use scratch memory
(register spills) and none may exceed the 160 KiB of LDS of a compute unit.

Spills are more than a speed matter here. The kernels order their direct-to-LDS copies by
counting outstanding vector-memory instructions (s_waitcnt vmcnt(n)); a spill store completes
out of order with respect to loads and would make such a count pass early, and a spill reload
makes the compiler wait for every copy in flight. The check compiles the kernel files for
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
    with concurrent.futures.ThreadPoolExecutor(4) as ex:
        parts = list(ex.map(resource_remarks, ["fa_fwd.hip", "fa_bwd.hip", "fa_d256.hip", "fa_fp8.hip", "fa_decode.hip"]))
    return {k: v for part in parts for k, v in part.items()}


def test_every_kernel_was_seen(remarks):
    names = " ".join(remarks)
    for k in ("fwd_kernel", "fwd_chain_kernel", "fwd_merge_kernel", "bwd_prep_kernel", "bwd_dkdv_kernel", "bwd_dq_kernel",
              "fwd256_kernel", "dkdv256_kernel", "dq256_kernel", "fwd_fp8_kernel", "keyless_rows_kernel"):
        assert k in names
    assert len(remarks) >= 60  # every instantiation reports


def test_no_kernel_spills_or_uses_scratch(remarks):
    bad = {k: v for k, v in remarks.items() if v.get("ScratchSize [bytes/lane]", 0) or v.get("VGPRs Spill", 0)}
    assert not bad, bad


def test_lds_fits_a_compute_unit(remarks):
    assert max(v.get("LDS Size [bytes/block]", 0) for v in remarks.values()) <= 160 * 1024


# ---- registers that a hand-issued load is still filling must not be touched
#
# fwd_chain_kernel reloads its Q_i operand registers with loads the compiler does not know to be
# loads (load16_async) and uses them only after a hand-written wait, through landed(). That is
# sound only if the compiler emits nothing between the two that reads or writes those registers:
# no copy, no spill, no reuse. The check below walks the compiler's assembly: from every such
# load, along every path of the control-flow graph, until the matching "landed" marker, and
# reports any instruction that names one of the load's registers. Two exceptions, both reachable
# only on paper, through the back edge of the loop over blocks: the MFMAs (the load is issued
# after the item's last score product, and the next item's first one comes after the marker) and
# the same load in another copy of the loop body.

def kernel_assembly(source):
    cmd = [fa_build.hipcc(), *[f for f in fa_build.FLAGS if f not in ("-shared", "-fPIC")], "--cuda-device-only", "-S",
           "-o", "-", os.path.join(fa_build.CSRC, source)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    kernels, name, body = {}, None, []
    for line in r.stdout.splitlines():
        m = re.match(r"^(_Z\w+):", line)
        if m:
            name, body = m.group(1), []
            kernels[name] = body
        elif name is not None:
            body.append(line)
            if line.strip().startswith("s_endpgm"):
                name = None
    return kernels


def vgprs(text):
    text = text.split(";")[0] if not text.lstrip().startswith(";") else text
    regs = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]", text):
        regs.update(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in re.finditer(r"\bv(\d+)\b", text):
        regs.add(int(m.group(1)))
    return regs


def touched_in_flight(lines):
    """[(load line, offending line)] for one kernel's assembly."""
    labels = {m.group(1): i for i, l in enumerate(lines) if (m := re.match(r"^(\.LBB\w+):", l))}
    in_asm, loads = False, []
    for i, l in enumerate(lines):
        t = l.strip()
        if t.startswith(";;#ASMSTART"):
            in_asm = True
        elif t.startswith(";;#ASMEND"):
            in_asm = False
        elif in_asm and t.startswith("global_load_dwordx4"):
            loads.append(i)

    def successors(i):
        t = lines[i].strip()
        if t.startswith("s_endpgm"):
            return []
        m = re.match(r"s_(c?branch\w*)\s+(\.LBB\w+)", t)
        if m:
            return [labels[m.group(2)]] + ([i + 1] if m.group(1).startswith("cbranch") else [])
        return [i + 1]

    bad = []
    for ld in loads:
        regs = vgprs(lines[ld].split(",")[0])  # the destination
        assert len(regs) == 4
        seen, todo = set(), successors(ld)
        while todo:
            i = todo.pop()
            if i in seen or i >= len(lines):
                continue
            seen.add(i)
            t = lines[i].strip()
            if t.startswith("; landed") and regs <= vgprs(t):
                continue  # this path has reached the marker
            is_code = t and not t.startswith((";", ".")) and not re.match(r"^\.?\w+:", t)
            if i in loads and regs == vgprs(t.split(",")[0]):
                continue  # the same reload in another copy of the loop body (the compiler peels iterations)
            if is_code and regs & vgprs(t) and not t.startswith("v_mfma"):
                bad.append((lines[ld].strip(), f"{i}: {t}"))
            todo.extend(successors(i))
    return loads, bad


def test_registers_of_loads_in_flight_are_left_alone():
    kernels = kernel_assembly("fa_fwd.hip")
    chained = {k: v for k, v in kernels.items() if "fwd_chain_kernel" in k}
    assert len(chained) == 4
    for name, lines in chained.items():
        loads, bad = touched_in_flight(lines)
        assert len(loads) >= 16, name  # the Q_i reload of both wave groups
        assert not bad, (name, bad[:5])


def test_the_in_flight_check_sees_a_planted_copy():
    lines = [
        ";;#ASMSTART", "global_load_dwordx4 v[8:11], v[2:3], off offset:0", ";;#ASMEND",
        "s_cbranch_scc1 .LBB0_2",
        "v_add_f32_e32 v1, v2, v3",
        ".LBB0_2:",
        "v_mov_b32_e32 v20, v9",
        ";;#ASMSTART", "; landed v[8:11]", ";;#ASMEND",
        "v_mov_b32_e32 v21, v9",
        "s_endpgm",
    ]
    loads, bad = touched_in_flight(lines)
    assert len(loads) == 1 and len(bad) == 1 and "v20" in bad[0][1]
