"""Builds libpreft.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libpreft.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # scalar fp32 code only: no packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def sources():
    """preft_api.hip (the C ABI, the launch logic and the few kernels it instantiates itself), slots.hip, and
    the kernel instantiations of csrc/instances/ (written by csrc/gen_instances.py)."""
    inst = os.path.join(CSRC, "instances")
    groups = sorted(os.path.join(inst, n) for n in os.listdir(inst) if n.endswith(".hip")) if os.path.isdir(inst) else []
    return [os.path.join(CSRC, "preft_api.hip"), os.path.join(CSRC, "slots.hip")] + groups


def build_library(verbose: bool = False) -> str:
    """Compile every HIP source (one hipcc per translation unit, in parallel) and link them into
    paper_2605_14217_amd/libpreft.so; returns its path."""
    import concurrent.futures
    import tempfile
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    compile_flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    jobs = max(1, min(len(sources()), int(os.environ.get("MAX_JOBS", "0")) or os.cpu_count() or 1, 16))
    messages = []

    def run(cmd):
        proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
        if proc.returncode != 0:
            raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + out)
        if out.strip():
            messages.append(out)

    with tempfile.TemporaryDirectory(prefix="preft_build_") as tmpdir:
        objects = [os.path.join(tmpdir, f"{i}_{os.path.basename(src)}.o") for i, src in enumerate(sources())]
        with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as pool:
            list(pool.map(lambda so: run([hipcc] + compile_flags + ["-c", so[0], "-o", so[1]]), zip(sources(), objects)))
        tmp = LIB_PATH + f".{os.getpid()}.tmp"
        run([hipcc] + HIPCC_FLAGS + objects + ["-o", tmp])
    if verbose and messages:
        print("\n".join(messages))
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
