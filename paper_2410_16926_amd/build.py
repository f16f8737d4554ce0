"""Builds libpvq.so (host code + gfx950 kernels) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_CSRC = os.path.join(_HERE, "csrc")
_INC = os.path.join(os.path.dirname(_HERE), "include")
LIB_PATH = os.path.join(_HERE, "libpvq.so")

SOURCES = ["pvq_host.cpp", "pvq_fast8_tables.cpp", "pvq_kernels.hip", "pvq_fast8.hip",
           "pvq_encode8.hip", "pvq_size_table.hip", "pvq_hadamard.hip", "pvq_wide.hip", "pvq_correct.hip", "pvq_walk.hip"]

# -ffp-contract=off: the encoder's float32 results are part of the format (no fused multiply-adds
# unless written as fmaf); correctly rounded float32 division and square root likewise.
# The target-feature pair keeps the compiler from forming packed float32 instructions.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt", "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return [os.path.join(_CSRC, s) for s in SOURCES]


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    deps = sources() + [os.path.join(_CSRC, "pvq_internal.h"), os.path.join(_CSRC, "pvq_fast8.h"),
                        os.path.join(_CSRC, "pvq_hadamard_dev.h"), os.path.join(_CSRC, "pvq_quantize_dev.h"),
                        os.path.join(_CSRC, "pvq_diagnostics.h"), os.path.join(_CSRC, "pvq_small_table.h"), os.path.join(_CSRC, "pvq_walk.h"),
                        os.path.join(_INC, "pvq.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def _run(cmd):
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + err)
    return err


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile the library: every source to an object of its own (side by side), then one link.
    Always compiles unless force=False and the library is up to date."""
    if not force and not is_stale():
        return LIB_PATH
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(_HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    compile_flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    jobs = []
    for src in sources():
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        jobs.append((obj, [hipcc, *compile_flags, "-x", "hip", f"-I{_INC}", f"-I{_CSRC}", "-c", src, "-o", obj]))
    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as pool:
        errs = list(pool.map(lambda j: _run(j[1]), jobs))
    errs.append(_run([hipcc, "--offload-arch=gfx950", "-fPIC", "-shared", "-o", LIB_PATH, *[j[0] for j in jobs]]))
    if verbose:
        print("\n".join(e for e in errs if e.strip()))
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
