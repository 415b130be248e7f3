"""Compile libcbm.so (HIP kernels + host builder + C ABI) for gfx950, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libcbm.so")
SOURCES = ["cbm_api.cpp", "cbm_builder.cpp", "cbm_kernels.hip", "cbm_gemm.hip", "cbm_build_kernels.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
COMMON = ["-O3", "-std=c++17", "-fPIC", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-Wall", "-Wno-unused-result", "-Wno-unused-value"]
# packed-fp32 VALU forms are kept out of all device code
DEVICE = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


# the compiler's per-kernel resource report: a kernel variant that spills registers fails the build (one register over
# the cap of a variant silently costs a quarter of its occupancy, or puts scratch traffic into a gather loop)
RESOURCES = ["-Rpass-analysis=kernel-resource-usage"]


def _spills(report: str, scratch_too: bool):
    """(kernel, what) for every kernel of a resource report with spilled registers (or, scratch_too, any scratch frame:
    the product kernels keep nothing in private memory; the builder's candidate search keeps its shortlist there)."""
    bad, name = [], None
    for ln in report.splitlines():
        if "remark:" not in ln:
            continue
        text = ln.split("remark:", 1)[1].strip()
        if text.startswith("Function Name:"):
            name = text.split(":", 1)[1].split("[")[0].strip()
        for key in ("SGPRs Spill:", "VGPRs Spill:") + (("ScratchSize [bytes/lane]:",) if scratch_too else ()):
            if text.startswith(key) and int(text[len(key):].split("[")[0].strip()) != 0:
                bad.append((name, text.split("[-R")[0].strip()))
    return bad


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(" ".join(cmd) + "\n" + r.stdout + r.stderr)
        raise RuntimeError("build failed: " + os.path.basename(cmd[-3] if len(cmd) > 3 else cmd[0]))
    out = r.stdout + r.stderr
    bad = _spills(out, scratch_too=not any("cbm_build_kernels" in a for a in cmd))
    if bad:
        sys.stderr.write("\n".join(f"{k}: {w}" for k, w in bad) + "\n")
        raise RuntimeError(f"build failed: {len(bad)} register spills in " + os.path.basename(cmd[-3]))
    warn, skip = [], 0
    for ln in out.splitlines():   # drop the resource remarks (and the source lines they quote) and the packed-fp32 note
        if "-Rpass-analysis=kernel-resource-usage" in ln:
            skip = 2 if "Function Name" in ln else 0
            continue
        if skip > 0:
            skip -= 1
            continue
        if "packed-fp32-ops" not in ln and "remarks generated" not in ln and ln.strip():
            warn.append(ln)
    if warn:
        sys.stderr.write("\n".join(warn) + "\n")


def build(verbose: bool = False) -> str:
    objdir = os.path.join(PKG, "_build")
    os.makedirs(objdir, exist_ok=True)
    objs = []
    cmds = []
    for src in SOURCES:
        obj = os.path.join(objdir, src + ".o")
        objs.append(obj)
        flags = COMMON + (DEVICE + RESOURCES if src.endswith(".hip") else [])
        cmds.append([HIPCC] + flags + ["-c", os.path.join(CSRC, src), "-o", obj])
    with ThreadPoolExecutor(max_workers=4) as ex:
        list(ex.map(_run, cmds))
    _run([HIPCC, "-shared", "-fPIC"] + DEVICE + objs + ["-o", LIB, "-lpthread"])
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
