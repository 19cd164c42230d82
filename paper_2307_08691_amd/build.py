"""Build the gfx950 attention library in-tree with hipcc.

    python -m paper_2307_08691_amd.build

produces paper_2307_08691_amd/libfa_gfx950.so from csrc/*.hip. hipcc
cross-compiles for gfx950 without a GPU.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfa_gfx950.so")
SOURCES = ["fa_api.hip", "fa_fwd.hip", "fa_bwd.hip", "fa_d256.hip", "fa_fp8.hip", "fa_decode.hip", "fa_probe.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    raise RuntimeError("hipcc not found")


def _compile(source: str, obj: str) -> str:
    cmd = [hipcc(), *FLAGS, "-c", "-o", obj, os.path.join(CSRC, source)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the AMDGPU-only target feature and says so: harmless
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {source}:\n" + err)
    return err


def build(verbose: bool = False) -> str:
    """Compile every HIP source (in parallel, one object each) and link the shared library.
    Always recompiles."""
    import concurrent.futures
    import tempfile
    with tempfile.TemporaryDirectory(prefix="fa_build_") as tmp:
        objs = [os.path.join(tmp, s.replace(".hip", ".o")) for s in SOURCES]
        if verbose:
            print(" ".join([hipcc(), *FLAGS, "-c"]), *SOURCES, flush=True)
        with concurrent.futures.ThreadPoolExecutor(len(SOURCES)) as ex:
            for err in ex.map(_compile, SOURCES, objs):
                if verbose and err:
                    print(err, file=sys.stderr)
        r = subprocess.run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
