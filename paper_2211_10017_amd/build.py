"""Builds libmoe_wq.so (the C-ABI HIP library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libmoe_wq.so")
OBJ = os.path.join(HERE, "_build")
# The same library with every hand-counted wait for direct-to-LDS loads replaced by a wait for all loads
# (-DMOE_WAIT_ALL_LOADS): only the translation units of the tiled kernels differ.  tests/ compare the two.
LIB_WAITALL = os.path.join(HERE, "libmoe_wq_waitall.so")
TILED = ["moe_ffn_tiled_4.hip", "moe_ffn_tiled_4_exact.hip", "moe_ffn_tiled_8.hip", "moe_ffn_tiled_8_exact.hip"]

SOURCES = ["moe_errors.hip", "moe_quantize.hip", "moe_gate.hip", "moe_permute.hip", "moe_ffn.hip", "moe_ffn_tiled.hip", "moe_ffn_tiled_4.hip", "moe_ffn_tiled_4_exact.hip",
           "moe_ffn_tiled_8.hip", "moe_ffn_tiled_8_exact.hip", "moe_ffn_stream.hip", "moe_ffn_decode.hip",
           "moe_combine.hip"]

# packed-fp32 VALU forms are switched off for every translation unit of this library
HIPCC_FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-I" + INCLUDE, "-I" + CSRC,
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _compile(src: str, variant: str = "") -> str:
    obj = os.path.join(OBJ, src.replace(".hip", variant + ".o"))
    extra = ["-DMOE_WAIT_ALL_LOADS"] if variant else []
    cmd = [_hipcc(), *HIPCC_FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, err))
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build_library(jobs: int = 8) -> str:
    """Compile every source and link the shared library; always recompiles."""
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        plain = pool.map(_compile, SOURCES)
        waitall = pool.map(lambda s: _compile(s, "_waitall"), TILED)
        objs, objs_waitall = list(plain), dict(zip(TILED, waitall))
    subprocess.check_call([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    other = [objs_waitall.get(src, obj) for src, obj in zip(SOURCES, objs)]
    subprocess.check_call([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_WAITALL, *other])
    return LIB


def build_ceilings() -> str:
    """Compile the stand-alone study programs under microbench/: the chip's achievable ceilings and the
    time-stamped decode kernel."""
    flags = [f for f in HIPCC_FLAGS if f != "-fPIC"]
    exe = ""
    for name, extra in (("ceilings", []), ("decode_timeline", [os.path.join(CSRC, "moe_errors.hip")])):
        src = os.path.join(HERE, "microbench", name + ".hip")
        exe = os.path.join(HERE, "microbench", name)
        res = subprocess.run([_hipcc(), *flags, src, *extra, "-o", exe], capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed for %s.hip:\n%s" % (name, res.stderr))
    return exe


if __name__ == "__main__":
    print(build_library())
    print(build_ceilings())
