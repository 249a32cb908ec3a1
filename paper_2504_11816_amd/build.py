"""Builds libokv.so (HIP, gfx950) next to this file with hipcc."""
import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libokv.so")
SOURCES = ["okv_kernels.hip", "okv_layer.hip", "okv_api.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fno-gpu-rdc",
         # keep the compiler from forming packed-fp32 instructions
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # matrix-core results stay in ordinary vector registers: the kernels here run one or two
         # wavefronts per SIMD and have registers to spare, and the accumulator-register form cost the
         # attention loop a copy of all 32 accumulators in and out per tile
         "-mllvm", "-amdgpu-mfma-vgpr-form",
         # the leading scalar and pointer arguments of a kernel arrive in scalar registers with the wavefront
         # instead of through a first round trip to the argument segment
         "-mllvm", "-amdgpu-kernarg-preload-count=14",
         "-Wall", "-Wno-unused-command-line-argument"]


def hipcc():
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: the okv library cannot be built")
    return exe


def build_library(verbose=False):
    """Compile every HIP source into libokv.so; always recompiles."""
    cmd = [hipcc(), *FLAGS, "-I", os.path.join(os.path.dirname(HERE), "include"),
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB + ".tmp"]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stdout + proc.stderr)
    if verbose and proc.stderr.strip():
        print(proc.stderr)
    os.replace(LIB + ".tmp", LIB)
    return LIB


MODEL_LIB = os.path.join(HERE, "libinfersave.so")


def build_model_library(verbose=False):
    """Compile the host-only selection model (plain C) into libinfersave.so; always recompiles."""
    gcc = shutil.which("gcc")
    if not gcc:
        raise RuntimeError("gcc not found: the selection-model library cannot be built")
    cmd = [gcc, "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra", "-I", os.path.join(os.path.dirname(HERE), "include"),
           os.path.join(CSRC, "infersave.c"), "-lm", "-o", MODEL_LIB + ".tmp"]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("gcc failed:\n" + proc.stdout + proc.stderr)
    if verbose and proc.stderr.strip():
        print(proc.stderr)
    os.replace(MODEL_LIB + ".tmp", MODEL_LIB)
    return MODEL_LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_model_library(verbose=True))
