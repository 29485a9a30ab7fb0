"""Builds ``libape_hip.so`` (the C-ABI attention library; depends on the HIP runtime only) and
``libape_layer.so`` (whole layers around it; links rocBLAS and libape_hip.so) and ``libape_probe.so``
(microbenchmarks of the box's ceilings for bench.py) for gfx950 with hipcc.

Usage: ``python -m paper_2502_05431_amd.build`` (cross-compiles without a GPU).
"""
from __future__ import annotations

import glob
import json
import os
import re
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libape_hip.so")
LAYER_LIB = os.path.join(PKG, "libape_layer.so")
PROBE_LIB = os.path.join(PKG, "libape_probe.so")
RESOURCES = os.path.join(PKG, "_build", "kernel_resources.json")

# -packed-fp32-ops off: packed fp32 VALU forms are not used on the test machines.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wall", "-Wno-unused-function", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
               "-I", os.path.join(CSRC, "layer")]


# Per-file flags.  The flash kernels keep every MFMA accumulator in the vector registers (the
# scores feed vector instructions at once; copying them out of the accumulation registers would
# cost one instruction per score) and never produce NaNs on valid inputs (-inf only), which lets
# the maxima compile to bare v_max3.
EXTRA_FLAGS = {
    "ape_flash_mfma.hip": ["-fno-honor-nans", "-mllvm", "-amdgpu-mfma-vgpr-form=1"],
}


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def layer_sources():
    return sorted(glob.glob(os.path.join(CSRC, "layer", "*.hip")))


def probe_sources():
    return sorted(glob.glob(os.path.join(CSRC, "probe", "*.hip")))


_REMARK = re.compile(r"remark:\s+(Function Name|VGPRs|AGPRs|ScratchSize \[bytes/lane\]|Occupancy \[waves/SIMD\]|"
                     r"LDS Size \[bytes/block\]|SGPRs): (\S+)")


def parse_resources(compiler_output: str) -> dict:
    """Per-kernel register, scratch and LDS use from hipcc's kernel-resource-usage remarks."""
    res, cur = {}, None
    for line in compiler_output.splitlines():
        m = _REMARK.search(line)
        if not m:
            continue
        key, val = m.group(1), m.group(2)
        if key == "Function Name":
            cur = res.setdefault(val, {})
        elif cur is not None:
            cur[key.split(" [")[0]] = int(val)
    return res


def build(verbose: bool = True, extra=()) -> str:
    objs = []
    procs = []
    layer_objs = []
    probe_objs = []
    for src in sources() + layer_sources() + probe_sources():
        obj = os.path.join(PKG, "_build", os.path.basename(src) + ".o")
        os.makedirs(os.path.dirname(obj), exist_ok=True)
        cmd = ["hipcc", *[f for f in HIPCC_FLAGS if f != "-shared"], *EXTRA_FLAGS.get(os.path.basename(src), []),
               "-Rpass-analysis=kernel-resource-usage", *extra, "-c", src, "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        (layer_objs if os.path.dirname(src).endswith("layer") else probe_objs if os.path.dirname(src).endswith("probe") else objs).append(obj)
    failed = False
    resources = {}
    for src, p in procs:
        out, _ = p.communicate()
        resources[os.path.basename(src)] = parse_resources(out)
        lines = [l for l in out.splitlines() if "packed-fp32-ops" not in l and "-Rpass-analysis" not in l
                 and "remark:" not in l]
        if p.returncode != 0:
            failed = True
        if verbose and lines:
            print("\n".join(lines))
    if failed:
        raise RuntimeError("hipcc failed")
    tmp = LIB + ".tmp%d" % os.getpid()
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
    os.replace(tmp, LIB)
    # the layer library finds the attention library next to itself ($ORIGIN)
    tmp = LAYER_LIB + ".tmp%d" % os.getpid()
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *layer_objs,
                           "-L" + PKG, "-lape_hip", "-Wl,-rpath,$ORIGIN", "-lrocblas"])
    os.replace(tmp, LAYER_LIB)
    # the probes of the box's ceilings (bench.py): on their own
    tmp = PROBE_LIB + ".tmp%d" % os.getpid()
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *probe_objs])
    os.replace(tmp, PROBE_LIB)
    with open(RESOURCES, "w") as f:
        json.dump(resources, f, indent=1, sort_keys=True)
    return LIB


if __name__ == "__main__":
    print(build(extra=sys.argv[1:]))
