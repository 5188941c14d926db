"""Build libkda.so (HIP, gfx950) in-tree with hipcc.

Run as ``python -m paper_2510_26692_amd.build``.  The library is built next to
this file so that it travels with the source tree; nothing is installed.
"""
import glob
import json
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libkda.so")
# What the compiler reports per kernel (registers, scratch bytes per lane, spills), written beside the library
# by every build; tests/test_kernel_resources.py reads it.
RESOURCES = os.path.join(HERE, "libkda.resources.json")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Wall", "-Wno-unused-function",
    # packed-fp32 instruction selection is switched off on purpose (known-bad forms)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # one remark per kernel with its register, scratch and spill figures (parsed below)
    "-Rpass-analysis=kernel-resource-usage",
]

_REMARK = re.compile(r"remark:\s+(Function Name|TotalSGPRs|VGPRs|AGPRs|ScratchSize \[bytes/lane\]|SGPRs Spill|VGPRs Spill"
                     r"|Occupancy \[waves/SIMD\]|LDS Size \[bytes/block\]|Dynamic Stack):\s+(\S+)")


def parse_resources(text):
    """{mangled kernel name: {figure: value}} from the compiler's kernel-resource-usage remarks."""
    out, cur = {}, None
    for m in _REMARK.finditer(text):
        key, val = m.group(1), m.group(2)
        if key == "Function Name":
            cur = out.setdefault(val, {})
        elif cur is not None:
            cur[key] = int(val) if val.lstrip("-").isdigit() else val
    return out


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def is_stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + glob.glob(os.path.join(CSRC, "*.h")) + \
        glob.glob(os.path.join(ROOT, "include", "*.h"))
    return any(os.path.getmtime(p) > t for p in deps)


def build(verbose=True, extra_flags=()):
    """Compile every HIP source into libkda.so; raises on failure."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + list(extra_flags) + \
        ["-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", tmp] + sources()
    if verbose:
        print(" ".join(cmd), flush=True)
    done = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    # the remarks go to the report, everything else the compiler said to the terminal
    noise = ("kernel-resource-usage", "is not a recognized feature for this target")
    rest = [ln for ln in done.stderr.splitlines() if not any(n in ln for n in noise)]
    if rest and (verbose or done.returncode != 0):
        print("\n".join(rest), file=sys.stderr, flush=True)
    if done.returncode != 0:
        if os.path.exists(tmp):
            os.remove(tmp)
        raise subprocess.CalledProcessError(done.returncode, cmd)
    os.replace(tmp, LIB)
    with open(RESOURCES, "w") as f:
        json.dump(parse_resources(done.stderr), f, indent=1, sort_keys=True)
    return LIB


if __name__ == "__main__":
    build(extra_flags=sys.argv[1:])
