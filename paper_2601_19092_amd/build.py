"""Builds the HIP library in-tree:  python -m paper_2601_19092_amd.build

One shared object, gfx950 only.  The flag pair after -Xclang switches off packed-fp32 code
generation (hipcc's host pass warns that it does not know the feature; that is harmless)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libaxe_hip.so")
SOURCES = ["api.cpp", "host_layout.cpp", "layout_algebra.cpp", "describe.cpp", "kernels_layout.hip", "kernels_gemm_small.hip",
           "kernels_gemm_bf16.hip", "kernels_gemm_grouped_stream.hip", "kernels_gemm_fp8.hip", "kernels_gemm_fp8_e8m0.hip"]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def build_library(verbose: bool = False, extra_flags=(), lib: str = LIB, objdir: str = "_build") -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    os.makedirs(os.path.join(HERE, objdir), exist_ok=True)
    for src in SOURCES:
        obj = os.path.join(HERE, objdir, src + ".o")
        cmd = [hipcc, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
        if p.returncode != 0:
            failed = True
            print(f"--- {src} failed:\n{out}", file=sys.stderr)
        elif verbose and out.strip():
            print(f"--- {src}:\n{out}")
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]
    subprocess.check_call(cmd)
    return lib


PARANOID_LIB = os.path.join(HERE, "libaxe_hip_paranoid.so")


def build_paranoid() -> str:
    """Checking build of the whole library (-DAXE_PARANOID: a full wait after every load into LDS and every store, a
    full wait and a workgroup barrier after every row of MFMAs in the large-tile GEMM kernels).  Loaded by one GPU
    test only, which requires its results to be bit-identical to the fast build's."""
    return build_library(extra_flags=("-DAXE_PARANOID",), lib=PARANOID_LIB, objdir="_build_paranoid")


def build_hostcheck() -> str:
    """Test-only library: the host layer linked against host-memory stand-ins of the integer
    kernels (csrc/cpu_emulation.cpp) so that planning can be checked without a GPU."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = os.path.join(HERE, "libaxe_hostcheck.so")
    srcs = [os.path.join(CSRC, f) for f in ("api.cpp", "host_layout.cpp", "layout_algebra.cpp", "describe.cpp", "cpu_emulation.cpp")]
    cmd = [hipcc, "-O1", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared", "-x", "hip",
           "-Wno-unused-command-line-argument", *srcs, "-o", out]
    subprocess.check_call(cmd)
    return out


def sanitizer_runtime() -> str:
    """The shared AddressSanitizer runtime of the compiler hipcc drives (preloaded into the process that loads the
    sanitized host library)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    return subprocess.check_output([hipcc, "-print-file-name=libclang_rt.asan-x86_64.so"], text=True).strip()


def build_hostcheck_sanitized() -> str:
    """Test-only library: build_hostcheck()'s sources with AddressSanitizer and UndefinedBehaviorSanitizer on the
    host side (the device pass has nothing to compile in these files).  tests/test_host_sanitizers.py runs the CPU
    tests of the host layer against it in a child process."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = os.path.join(HERE, "libaxe_hostcheck_san.so")
    srcs = [os.path.join(CSRC, f) for f in ("api.cpp", "host_layout.cpp", "layout_algebra.cpp", "describe.cpp", "cpu_emulation.cpp")]
    cmd = [hipcc, "-O1", "-g", "-fno-omit-frame-pointer", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared", "-x", "hip",
           "-Wno-unused-command-line-argument", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", *srcs, "-o", out]
    subprocess.check_call(cmd)
    return out


def build_probe() -> str:
    """Measurement aids (csrc/probes.hip): register-only MFMA loops, loaded by bench.py --ceilings only."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = os.path.join(HERE, "libaxe_probe.so")
    subprocess.check_call([hipcc, *FLAGS, "-shared", os.path.join(CSRC, "probes.hip"), "-o", out], stderr=subprocess.DEVNULL)
    return out


if __name__ == "__main__":
    print(build_library(verbose="-v" in sys.argv))
    print(build_paranoid())
    print(build_hostcheck())
    print(build_hostcheck_sanitized())
    print(build_probe())
