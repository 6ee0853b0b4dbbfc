"""Builds libstartrail.so (gfx950) in-tree with hipcc.

    python paper_2407_00611_amd/build.py      (run as a script: importing the package needs the built library)

Every source is compiled on every call; objects go to ``_build/`` (git-ignored).
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
OUT = os.path.join(PKG, "libstartrail.so")
OBJ_DIR = os.path.join(PKG, "_build")

SOURCES = ["st_api.cpp", "st_runtime.cpp", "st_f32.hip", "st_elementwise.hip", "st_fwd_bf16.hip", "st_bwd_bf16.hip", "st_bwd_dkv_fast.hip", "st_bwd_dq_fast.hip", "st_fwd_fast.hip", "st_probe.hip"]
# assembly main loops written out by generator scripts before compiling: (script, output)
GENERATED = [("gen_bwd_dkv_asm.py", "st_bwd_dkv_asm.inc"), ("gen_bwd_dq_asm.py", "st_bwd_dq_asm.inc"),
             ("gen_fwd_asm.py", "st_fwd_asm.inc"), ("gen_fwd_asm.py 64", "st_fwd64_asm.inc"),
             ("gen_bwd_dq_asm.py 64", "st_bwd_dq64_asm.inc"), ("gen_bwd_dkv_asm.py 64", "st_bwd_dkv64_asm.inc"),
             ("gen_probe_asm.py", "st_probe_asm.inc")]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-fp32 VALU forms (v_pk_add_f32, v_pk_mul_f32, v_pk_fma_f32) are switched off for device code on purpose:
# some of their forms have given wrong results on the target machines
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, "-x", "hip", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout}\n{r.stderr}")
    noise = "packed-fp32-ops' is not a recognized feature"
    warn = "\n".join(l for l in r.stderr.splitlines() if l.strip() and noise not in l)
    if warn:
        sys.stderr.write(warn + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    for script, out in GENERATED:
        name, *args = script.split()
        r = subprocess.run([sys.executable, os.path.join(CSRC, name), *args], capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"{script} failed:\n{r.stderr}")
        with open(os.path.join(CSRC, out), "w") as f:
            f.write(r.stdout)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", *objs, "-L/opt/rocm/lib", "-lhsa-runtime64", "-o", OUT]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"built {OUT}")
    return OUT


if __name__ == "__main__":
    build()
