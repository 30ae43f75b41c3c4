"""Writes csrc/instances/: the kernel instantiations of libpreft.so spread over several translation units.

preft_api.hip uses some 250 instantiations of the tile kernels; in one translation unit that is minutes
of compile time.  This script asks the compiler which instantiations preft_api.hip needs (its
kernel-resource-usage remarks, with the extern declarations switched off), deals them out to a few
instances/group_<k>.hip files as explicit instantiations, and lists them all in
instances/extern_kernels.inc as `extern template` declarations, which preft_api.hip includes: it then
only launches them.  build.py compiles the groups in parallel.  An instantiation that is missing from
the lists (someone added a launch and did not run this script) is simply compiled in preft_api.hip as
before: the lists are an optimisation of the build, not a registry.

Run from the repository root after adding or removing a kernel instantiation:
    python paper_2605_14217_amd/csrc/gen_instances.py
"""
from __future__ import annotations

import os
import re
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
OUT = os.path.join(HERE, "instances")
GROUPS = 7
FAMILIES = {            # kernel template -> (header, rough relative compile cost)
    "preft::mfma_wide_kernel": ("mfma_wide_kernel.hpp", 3),
    "preft::mfma_wide_layers_kernel": ("mfma_wide_kernel.hpp", 3),
    "preft::mfma_expand_panel_kernel": ("mfma_wide_kernel.hpp", 1),
    "preft::mfma_tile_kernel": ("mfma_kernel.hpp", 2),
    "preft::mfma_tile_layers_kernel": ("mfma_kernel.hpp", 2),
    "preft::valu_tile_kernel": ("valu_kernel.hpp", 1),
    "preft::valu_tile_layers_kernel": ("valu_kernel.hpp", 1),
}


def needed_instantiations():
    from paper_2605_14217_amd.build import HIPCC_FLAGS
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    cmd = [hipcc] + flags + ["-DPREFT_NO_EXTERN_KERNELS", "--cuda-device-only", "-c", os.path.join(HERE, "preft_api.hip"),
                             "-o", os.devnull, "-Rpass-analysis=kernel-resource-usage"]
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError(proc.stdout[-4000:])
    mangled = sorted(set(re.findall(r"Function Name: (\S+)", proc.stdout)))
    demangled = subprocess.run(["c++filt"], input="\n".join(mangled), stdout=subprocess.PIPE, text=True, check=True).stdout.splitlines()
    out = []
    for d in demangled:
        m = re.match(r"void (preft::\w+)<(.*)>\((.*)\)$", d.strip())
        if m and m.group(1) in FAMILIES:
            out.append((m.group(1), m.group(2), m.group(3)))
    return out


def main():
    inst = needed_instantiations()
    os.makedirs(OUT, exist_ok=True)
    for name in os.listdir(OUT):
        os.remove(os.path.join(OUT, name))
    bins = [[] for _ in range(GROUPS)]
    load = [0] * GROUPS
    for item in sorted(inst, key=lambda it: -FAMILIES[it[0]][1]):       # greedy: heaviest first into the lightest bin
        k = load.index(min(load))
        bins[k].append(item)
        load[k] += FAMILIES[item[0]][1]
    note = "// written by gen_instances.py: do not edit by hand\n"
    with open(os.path.join(OUT, "extern_kernels.inc"), "w") as f:
        f.write(note + "// kernel instantiations that instances/group_*.hip define: preft_api.hip only launches them\n")
        for name, targs, params in sorted(inst):
            f.write(f"extern template __global__ void {name}<{targs}>({params});\n")
    for k, items in enumerate(bins):
        headers = sorted({FAMILIES[name][0] for name, _, _ in items})
        with open(os.path.join(OUT, f"group_{k}.hip"), "w") as f:
            f.write(note + "".join(f'#include "../{h}"\n' for h in headers) + "\n")
            for name, targs, params in sorted(items):
                f.write(f"template __global__ void {name}<{targs}>({params});\n")
    print(f"{len(inst)} instantiations in {GROUPS} groups (weights {load})")


if __name__ == "__main__":
    import sys
    sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
    main()
