"""Build libssn_hip.so (the C-ABI library of include/ssn.h) for gfx950 with hipcc, in-tree.

Next to the library the build leaves kernel_resources.json: registers and scratch bytes per lane of every
kernel, from the compiler's own resource remarks.  A kernel that uses scratch memory at all pays ~14 us per
launch on MI355X, so the test suite checks that none of this library's kernels does."""
import glob
import json
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libssn_hip.so")
RESOURCES = os.path.join(HERE, "kernel_resources.json")
SRCS = sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")))
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep the compiler from forming packed fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
]


def _resources(remarks):
    """{kernel: {"vgprs": .., "scratch": ..}} from -Rpass-analysis=kernel-resource-usage remarks."""
    out, name = {}, None
    for line in remarks.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            out[name] = {}
            continue
        if name is None:
            continue
        m = re.search(r" VGPRs: (\d+)", line)
        if m:
            out[name]["vgprs"] = int(m.group(1))
        m = re.search(r"ScratchSize \[bytes/lane\]: (\d+)", line)
        if m:
            out[name]["scratch"] = int(m.group(1))
    return out


def build(verbose=False):
    procs = []
    for src in SRCS:                      # every source at once: one long file dominates the build
        obj = src[:-4] + ".o"
        cmd = (["hipcc", "-c"] + [f for f in FLAGS if f != "-shared"]
               + ["-Rpass-analysis=kernel-resource-usage", "-o", obj, src])
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, obj, cmd, subprocess.Popen(cmd, stderr=subprocess.PIPE, text=True)))
    objs, resources = [], {}
    for src, obj, cmd, proc in procs:
        _, err = proc.communicate()
        if proc.returncode != 0:
            sys.stderr.write(err)
            raise subprocess.CalledProcessError(proc.returncode, cmd)
        resources[os.path.basename(src)] = _resources(err)
        objs.append(obj)
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    with open(RESOURCES, "w") as fh:
        json.dump(resources, fh, indent=0, sort_keys=True)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
    print(LIB)
