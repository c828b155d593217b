"""Builds libgear.so (the C-ABI HIP library) in-tree with hipcc for gfx950."""
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libgear.so")

SOURCES = ["gear_api.hip", "compress_filter.hip", "compress_values.hip", "lowrank.hip", "decode.hip", "decompress_export.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def kernel_resources(stderr_text):
    """{kernel symbol: {"vgprs": n, "scratch": bytes per lane}} from the compiler's resource remarks."""
    out, name = {}, None
    for line in stderr_text.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            out[name] = {}
            continue
        if name is None:
            continue
        m = re.search(r"VGPRs: (\d+)", line)
        if m and "vgprs" not in out[name]:
            out[name]["vgprs"] = int(m.group(1))
        m = re.search(r"ScratchSize \[bytes/lane\]: (\d+)", line)
        if m:
            out[name]["scratch"] = int(m.group(1))
    return out


def _compile(src):
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = ["hipcc", "-c", os.path.join(CSRC, src), "-o", obj, "-Rpass-analysis=kernel-resource-usage"] + FLAGS
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, r.stdout, r.stderr))
    # No kernel may spill registers to scratch memory.  This compiler has placed a
    # spill store inside a region where only some lanes were enabled and reloaded
    # the value for all lanes afterwards (stale data in the other lanes, wrong
    # addresses); a kernel without scratch cannot be hit by that.
    spilled = {k: v["scratch"] for k, v in kernel_resources(r.stderr).items() if v.get("scratch", 0) > 0}
    if spilled:
        raise RuntimeError("kernels in %s spill to scratch memory (bytes per lane): %s" % (src, spilled))
    return obj


def build_library(verbose=True):
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = ["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build_library()
