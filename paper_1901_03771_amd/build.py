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


SAN_LIB = os.path.join(HERE, "libgrumpy_hip_san.so")


def sanitizer_runtime() -> str:
    """The AddressSanitizer runtime of hipcc's own clang (what a process that loads SAN_LIB has to preload), or ""."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    r = subprocess.run([hipcc, "-print-file-name=libclang_rt.asan-x86_64.so"], stdout=subprocess.PIPE, stderr=subprocess.DEVNULL, text=True)
    path = r.stdout.strip()
    if r.returncode == 0 and os.path.isabs(path) and os.path.exists(path):
        return path
    import glob
    found = sorted(glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so"))
    return found[-1] if found else ""


def build_sanitized(verbose: bool = False) -> str:
    """The same library with its HOST code (recorder, planner, plan cache, code generator, runtime) instrumented by
    AddressSanitizer and UndefinedBehaviorSanitizer; device code is compiled as usual.  For the CPU-only checks that
    drive the host logic through a device-less context in dry-run mode (tests/test_sanitized_host.py): a process
    that loads it sets GRUMPY_HIP_LIB to the path returned and preloads sanitizer_runtime().  One compiler process
    per source file, in parallel."""
    import concurrent.futures
    import tempfile
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    common = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-ffp-contract=off",
              "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
              "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined"]
    with tempfile.TemporaryDirectory(prefix="grumpy_san_") as tmp:
        def compile_one(src):
            obj = os.path.join(tmp, src + ".o")
            r = subprocess.run(common + ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
            if r.returncode != 0:
                raise RuntimeError(f"hipcc failed on {src}:\n" + r.stdout)
            return obj
        with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
            objs = list(pool.map(compile_one, SOURCES))
        cmd = common + ["-shared", "-shared-libsan", "-o", SAN_LIB] + objs + ["-lhiprtc"]
        if verbose:
            print(" ".join(cmd))
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if r.returncode != 0:
            raise RuntimeError("linking the sanitized library failed:\n" + r.stdout)
    return SAN_LIB


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
    if "--sanitized" in sys.argv[1:]:
        print(build_sanitized(verbose=True))
    else:
        print(build(verbose=True))
