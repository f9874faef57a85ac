"""Build libhag.so (host C++ + HIP kernels for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libhag.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = [os.path.join(HERE, "csrc", f) for f in (
    "hag_host.cpp", "hag_seq.cpp", "hag_device.hip", "hag_search_device.hip", "hag_probe.hip", "hag_seq_device.hip",
    # the gather and component kernels are instantiated for many widths and roles: one unit per
    # element type (and reduction) so that they compile side by side
    "hag_gather_f32_sum.hip", "hag_gather_f32_max.hip", "hag_gather_i32_sum.hip", "hag_gather_i32_max.hip",
    "hag_component_f32.hip", "hag_component_i32.hip")]
HEADERS = [os.path.join(HERE, "csrc", f) for f in ("hag_internal.hpp", "hag_device_common.hpp", "hag_gather.inc",
                                                   "hag_component.inc")] + [os.path.join(ROOT, "include", "hag.h")]


def build_library(force: bool = True, verbose: bool = False) -> str:
    if not force and os.path.exists(LIB):
        newest = max(os.path.getmtime(p) for p in SOURCES + HEADERS)
        if os.path.getmtime(LIB) >= newest:
            return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    common = [
        hipcc, "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-Wall", "-Wno-unused-function", "-Rpass-analysis=kernel-resource-usage",
        "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(HERE, "csrc"),
    ]
    # one compiler process per source file, side by side; objects go to a build folder that is
    # not tracked
    os.makedirs(OBJ_DIR, exist_ok=True)
    objs = [os.path.join(OBJ_DIR, os.path.basename(src) + ".o") for src in SOURCES]
    procs = []
    for src, obj in zip(SOURCES, objs):
        cmd = [*common, "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd))
        procs.append((cmd, subprocess.Popen(cmd, stderr=subprocess.PIPE, text=True)))
    usage, failed = {}, None
    for cmd, pr in procs:
        _, err = pr.communicate()
        try:
            usage.update(check_resource_usage(err))
        finally:
            if pr.returncode != 0 and failed is None:
                failed = (pr.returncode, cmd)
    if failed:
        raise subprocess.CalledProcessError(*failed)
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB, "-lpthread"]
    if verbose:
        print(" ".join(link))
    subprocess.run(link, check=True)
    if verbose:
        for name, u in sorted(usage.items()):
            print(f"{name}: {u.get('VGPRs', '?')} VGPRs, {u.get('LDS Size [bytes/block]', '?')} B LDS")
    return LIB


def check_resource_usage(stderr: str) -> dict:
    """Parse the compiler's per-kernel resource remarks; print everything else it said.

    A kernel that touches scratch memory (register spills, or its argument block copied to the
    stack because of a run-time choice the optimiser could not resolve) runs several times slower
    without failing any test, so it fails the build instead."""
    usage, name, after_remark, held = {}, None, False, []
    for line in stderr.splitlines():
        if line.startswith("In file included from"):
            held.append(line)          # belongs to the diagnostic that follows; dropped if that is a remark
            continue
        if "[-Rpass-analysis=kernel-resource-usage]" not in line:
            for h in held:
                print(h, file=sys.stderr)
            held = []
            snippet = re.match(r"\s*(\d+\s*)?\|", line) is not None       # source excerpt under a diagnostic
            if not (snippet and after_remark) and "packed-fp32-ops" not in line and line.strip():
                print(line, file=sys.stderr)          # ordinary warnings and errors
            if not snippet:
                after_remark = False
            continue
        after_remark, held = True, []
        text = line.split("remark:", 1)[1].rsplit("[-Rpass", 1)[0].strip()
        if text.startswith("Function Name:"):
            name = text.split(":", 1)[1].strip()
            usage[name] = {}
        elif name and ":" in text:
            k, v = text.rsplit(":", 1)
            usage[name][k.strip()] = v.strip()
    bad = {n: u["ScratchSize [bytes/lane]"] for n, u in usage.items() if u.get("ScratchSize [bytes/lane]", "0") != "0"}
    if bad:
        raise RuntimeError("kernels that use scratch memory (bytes per lane): " + ", ".join(f"{n}: {b}" for n, b in bad.items()))
    return usage


if __name__ == "__main__":
    print(build_library(force=True, verbose=True))
