"""Builds synth/libddd_synth.so: the on-device workload generators and measurement kernels of the tests and
the benchmark (stand-in draft body and target model, round statistics, plain read stream, MFMA loop).  It is a
shared object of its own, linked against the product library, so that libddd.so holds the method only."""
from __future__ import annotations

import os
import subprocess

SYNTH_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(SYNTH_DIR, "libddd_synth.so")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build_library(product_lib: str, verbose: bool = True) -> str:
    """Compile synth/csrc and link it against the product library at `product_lib`; returns the path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    build_dir = os.path.join(SYNTH_DIR, "_build")
    os.makedirs(build_dir, exist_ok=True)
    obj = os.path.join(build_dir, "synth_workload.o")
    cmd = [hipcc] + FLAGS + ["-c", os.path.join(SYNTH_DIR, "csrc", "synth_workload.hip"), "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on synth_workload.hip:\n{out}")
    if verbose and out.strip():
        print(out)
    pdir = os.path.dirname(os.path.abspath(product_lib))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH, obj, "-L" + pdir, "-lddd",
           "-Wl,-rpath,$ORIGIN/" + os.path.relpath(pdir, SYNTH_DIR)]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB_PATH
