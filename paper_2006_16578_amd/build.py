"""Builds libbnn.so (HIP, gfx950 only) in-tree next to this file.

    python -m paper_2006_16578_amd.build [--force]

Each translation unit is compiled to an object in ``_build/`` and the objects are linked into
``libbnn.so``.  Objects are rebuilt when their source or any header is newer.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libbnn.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SOURCES = ["bnn_api.hip", "bnn_valu.hip", "bnn_mfma.hip", "bnn_mfma_conv_v4.hip", "bnn_mfma_conv_v2.hip",
           "bnn_mfma_conv_v1.hip", "bnn_mfma_conv_staged.hip", "bnn_aux.hip", "bnn_bwn.hip", "bnn_persistent.hip", "bnn_probe.hip", "bnn_mfma_skinny.hip", "bnn_mfma_wide.hip", "bnn_mfma_conv_patch.hip"]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Wall", "-Wno-unused-value",
         "-Rpass-analysis=kernel-resource-usage",   # per-kernel register / scratch report, scanned for spills below
         # packed fp32 VALU forms are kept off for every device function of this library
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _headers():
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    hs.append(os.path.join(os.path.dirname(HERE), "include", "bnn.h"))
    return hs


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    srcp = os.path.join(CSRC, src)
    newest = max(os.path.getmtime(p) for p in [srcp] + _headers())
    if force or not os.path.exists(obj) or os.path.getmtime(obj) < newest:
        cmd = [HIPCC] + FLAGS + ["-c", srcp, "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        lines = r.stderr.splitlines()
        if r.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s" % (src, "\n".join(l for l in lines if "remark:" not in l)))
        for l in lines:     # the resource-usage remarks are scanned below, not echoed
            if ("warning:" in l or "error:" in l) and "packed-fp32-ops" not in l and "target feature" not in l:
                sys.stderr.write(l + "\n")
        # a kernel that spills registers to scratch is a performance bug here: say so loudly
        name = "?"
        for l in lines:
            if "Function Name:" in l:
                name = l.split("Function Name:")[1].split("[")[0].strip()
            elif "VGPRs Spill:" in l and int(l.split("VGPRs Spill:")[1].split("[")[0]) > 0:
                sys.stderr.write("build.py: WARNING %s: kernel %s spills %s VGPRs\n"
                                 % (src, name, l.split("VGPRs Spill:")[1].split("[")[0].strip()))
    return obj


def build(force: bool = False, jobs: int = 8) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    if force or not os.path.exists(LIB) or any(os.path.getmtime(o) > os.path.getmtime(LIB) for o in objs):
        tmp = LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs)
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
