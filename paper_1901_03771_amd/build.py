"""Builds, in-tree, the C-ABI library libgrumpy_hip.so (hipcc, gfx950) and the CPython type with the
binding's recording fast paths (_fastbind, host C), then compiles the ahead-of-time kernel pack with the
library just built (hipRTC, no GPU needed)."""
from __future__ import annotations

import os
import subprocess
import sys
import sysconfig

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libgrumpy_hip.so")
SOURCES = ["recorder.cpp", "plan.cpp", "codegen.cpp", "runtime.cpp", "interp.cpp", "plancache.cpp", "stream_kernels.hip", "interp_kernel.hip", "static_scratch.hip"]


def build(verbose: bool = False, pack: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O2", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
           "-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES] + ["-lhiprtc"]
    if verbose:
        print(" ".join(cmd))
    # hipcc's host pass warns that it does not know the packed-fp32 feature: harmless, filtered
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "is not a recognized feature for this target" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    build_fastbind(verbose)
    if pack:
        build_pack(verbose)
    return LIB


def build_pack(verbose: bool = False) -> None:
    # in a process of its own: it has to load the library that was just built
    code = "from paper_1901_03771_amd import kernel_pack; kernel_pack.build_pack(verbose=%r)" % verbose
    env = dict(os.environ, PYTHONPATH=os.path.dirname(HERE) + os.pathsep + os.environ.get("PYTHONPATH", ""))
    r = subprocess.run([sys.executable, "-c", code], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("building the kernel pack failed:\n" + r.stdout)
    if verbose and r.stdout.strip():
        print(r.stdout)


def build_fastbind(verbose: bool = False) -> str:
    out = os.path.join(HERE, "_fastbind" + (sysconfig.get_config_var("EXT_SUFFIX") or ".so"))
    cmd = [os.environ.get("CC", "gcc"), "-O2", "-fPIC", "-shared", "-Wall", "-I" + sysconfig.get_paths()["include"],
           os.path.join(CSRC, "fastbind.c"), "-o", out]
    if verbose:
        print(" ".join(cmd))
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("building _fastbind failed:\n" + r.stdout)
    if verbose and r.stdout.strip():
        print(r.stdout)
    return out


if __name__ == "__main__":
    print(build(verbose=True))
