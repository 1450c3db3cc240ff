"""Builds libllma.so (HIP, gfx950 only) in-tree with hipcc.  No torch involved: the library
is a plain C-ABI shared object; the Python binding loads it with ctypes."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libllma.so")
SOURCES = ["kernels_bf16.hip", "kernels_f32.hip", "kernels_misc.hip", "llma_api.hip", "llma_noalloc.hip"]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Wno-unused-result",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = [_hipcc(), *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{out}")
    if out.strip():
        sys.stderr.write(out + "\n")
    return obj


# stand-alone measurement tool (csrc/microbench.hip): the same source twice, the second time with the
# per-wave time stamps compiled into the GEMM kernels
TOOLS = {"llma_microbench": [], "llma_microbench_timeline": ["-DMICROBENCH_TIMELINE"]}


def _tool(name: str) -> str:
    out = os.path.join(HERE, "tools", name)
    cmd = [_hipcc(), *[f for f in FLAGS if f != "-fPIC"], *TOOLS[name], os.path.join(CSRC, "microbench.hip"), "-o", out]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {name}:\n" + "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l))
    return out


def build(verbose: bool = True, tools: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    os.makedirs(os.path.join(HERE, "tools"), exist_ok=True)
    with ThreadPoolExecutor(max_workers=6) as ex:
        tool_jobs = [ex.submit(_tool, t) for t in TOOLS] if tools else []
        objs = list(ex.map(_compile, SOURCES))
        built_tools = [j.result() for j in tool_jobs]
    subprocess.check_call([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    if verbose:
        print(f"built {LIB}" + "".join(f"\nbuilt {t}" for t in built_tools))
    return LIB


if __name__ == "__main__":
    build(tools="--no-tools" not in sys.argv)
