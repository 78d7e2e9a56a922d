"""Compile the HIP sources under csrc/ into libsea_hip.so (in-tree) for gfx950."""
from __future__ import annotations

import concurrent.futures
import glob
import os
import subprocess
import tempfile

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libsea_hip.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    # keep the compiler from forming packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # MFMA accumulators stay in ordinary VGPRs (no copies to and from the AGPR half)
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + glob.glob(os.path.join(CSRC, "*.h")) + [os.path.join(_ROOT, "include", "sea.h")]
    return any(os.path.getmtime(f) > t for f in deps)


def build(verbose: bool = False) -> str:
    """Always recompiles: one hipcc per source file (in parallel), then one link.  Returns the
    path of the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    noise = "is not a recognized feature for this target"
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    inc = ["-I", os.path.join(_ROOT, "include"), "-I", CSRC]

    def run(cmd):
        res = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(ln for ln in res.stderr.splitlines() if noise not in ln)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + err)
        return err

    with tempfile.TemporaryDirectory(prefix="sea_build_") as tmp:
        jobs = [(src, os.path.join(tmp, os.path.basename(src) + ".o")) for src in sources()]
        workers = max(1, min(len(jobs), int(os.environ.get("MAX_JOBS", os.cpu_count() or 1))))
        with concurrent.futures.ThreadPoolExecutor(workers) as pool:
            logs = list(pool.map(lambda j: run([hipcc, *flags, *inc, "-c", j[0], "-o", j[1]]), jobs))
        logs.append(run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *[o for _, o in jobs]]))
    if verbose and any(l.strip() for l in logs):
        print("\n".join(l for l in logs if l.strip()))
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
