"""Build libsts.so (HIP, gfx950 only) in-tree with hipcc. No JIT, no torch extension machinery:
the library has a plain C ABI and is loaded with ctypes."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsts.so")
SOURCES = ["api.hip", "attn.hip", "select.hip", "headmap.hip", "scratch.hip", "union.hip"]
HEADERS = [os.path.join(CSRC, "common.h"), os.path.join(HERE, "..", "include", "sts.h")]

# -packed-fp32-ops is switched off on purpose: packed fp32 instructions are not to be
# generated for the test machines.
COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Rpass-analysis=kernel-resource-usage"]   # registers, spills and scratch of every kernel, kept beside the objects
RESOURCES = os.path.join(HERE, "_build", "kernel_resources.txt")
# selection must reproduce a fixed fp32 addition order bit for bit: no contraction there
PER_FILE = {"select.hip": ["-ffp-contract=off"]}


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def needs_build() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + HEADERS
    return any(os.path.getmtime(d) > t for d in deps)


def kernel_resources() -> dict:
    """{kernel symbol: {"VGPRs": n, "AGPRs": n, "ScratchSize": bytes per lane, "VGPRs Spill": n, ...}} of the
    last build, from the compiler's own remarks."""
    res, cur = {}, None
    with open(RESOURCES) as f:
        for ln in f:
            body = ln.split("remark:", 1)[1].rsplit("[-Rpass", 1)[0].strip()
            key, _, val = body.partition(":")
            key, val = key.strip(), val.strip()
            if key == "Function Name":
                cur = res.setdefault(val, {})
            elif cur is not None:
                key = key.split(" [")[0]
                cur[key] = int(val) if val.lstrip("-").isdigit() else val
    return res


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP source for gfx950 and link libsts.so next to this file."""
    if not force and not needs_build():
        return LIB
    hipcc = _hipcc()
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [hipcc, *COMMON, *PER_FILE.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    remarks = []
    for src, pr in procs:
        out, _ = pr.communicate()
        if pr.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        remarks += [ln for ln in out.splitlines() if "-Rpass-analysis=kernel-resource-usage" in ln]
        rest = "\n".join(ln for ln in out.splitlines() if "-Rpass-analysis=kernel-resource-usage" not in ln)
        if verbose and rest.strip():
            print(rest)
    with open(RESOURCES, "w") as f:
        f.write("\n".join(remarks) + "\n")
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose="-v" in sys.argv))
