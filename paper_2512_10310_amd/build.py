"""Builds libevl.so (HIP kernels + C ABI) for gfx950 in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libevl.so")
SOURCES = ["evl_kernels.hip", "evl_api.cpp"]
HEADERS = [os.path.join(CSRC, "evl_internal.h"), os.path.join(ROOT, "include", "evl.h")]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + HEADERS
    return any(os.path.getmtime(d) > t for d in deps)


def build(verbose: bool = False) -> str:
    """Compile every HIP source for gfx950 and link the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc, "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
               # packed fp32 ALU forms stay off (known-unreliable on the test machines)
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wall", "-Wno-unused-command-line-argument",
               "-I", os.path.join(ROOT, "include"), "-I", CSRC,
               "-c", os.path.join(CSRC, src), "-o", obj]
        if src.endswith(".hip"):
            cmd[1:1] = ["-x", "hip"]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(l for l in r.stdout.splitlines()
                        if "is not a recognized feature for this target" not in l)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, out))
        if out.strip() and verbose:
            print(out)
        objs.append(obj)
    tmp = LIB + ".tmp%d" % os.getpid()
    subprocess.check_call([hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp] + objs)
    os.replace(tmp, LIB)
    return LIB


def host_probe_is_stale() -> bool:
    probe_dir = os.path.join(ROOT, "tests", "host_probe")
    out = os.path.join(probe_dir, "libevl_probe.so")
    if not os.path.exists(out):
        return True
    deps = [os.path.join(CSRC, "evl_api.cpp"), os.path.join(probe_dir, "launch_probe.cpp")] + HEADERS
    return any(os.path.getmtime(d) > os.path.getmtime(out) for d in deps)


def build_host_probe(verbose: bool = False) -> str:
    """Test infrastructure, not part of the product: the library's host side (evl_api.cpp) linked
    with tests/host_probe/launch_probe.cpp, which checks kernel arguments instead of launching.
    Host code only, built with the undefined-behaviour sanitizer and checked std::vector indexing."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    probe_dir = os.path.join(ROOT, "tests", "host_probe")
    out = os.path.join(probe_dir, "libevl_probe.so")
    rt = os.path.dirname(subprocess.run([hipcc, "-print-file-name=libclang_rt.ubsan_standalone-x86_64.so"],
                                        stdout=subprocess.PIPE, text=True).stdout.strip())
    cmd = [hipcc, "-O1", "-g", "-std=c++17", "-fPIC", "-shared", "-Wall", "-D_GLIBCXX_ASSERTIONS",
           "-fno-gpu-sanitize", "-fsanitize=undefined", "-fno-sanitize-recover=all", "-shared-libsan",
           "-Wl,-rpath," + rt, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(CSRC, "evl_api.cpp"), os.path.join(probe_dir, "launch_probe.cpp"), "-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("building the host probe failed:\n" + r.stdout)
    return out


def build_peak_probe(verbose: bool = False) -> str:
    """bench.py's helper, a library of its own: csrc/peak_probe.hip (an MFMA-only loop that measures
    what the matrix pipes reach on this chip)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = os.path.join(PKG, "libevl_peakprobe.so")
    cmd = [hipcc, "-x", "hip", "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall",
           "-Wno-unused-command-line-argument", os.path.join(CSRC, "peak_probe.hip"), "-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("building the peak probe failed:\n" + r.stdout)
    return out


def build_lds_probe(verbose: bool = False) -> str:
    """Measurement helper, a program of its own: csrc/lds_patterns_probe.hip (the LDS access patterns of
    the attention kernel, one kernel per pattern, for a bank-conflict counter pass)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = os.path.join(PKG, "lds_patterns_probe")
    cmd = [hipcc, "-x", "hip", "-O3", "-std=c++17", "--offload-arch=gfx950", "-Wno-unused-value",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument", os.path.join(CSRC, "lds_patterns_probe.hip"), "-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("building the LDS probe failed:\n" + r.stdout)
    return out


def build_c_abi_test(verbose: bool = False) -> str:
    """Test infrastructure: tests/c_abi/closed_forms.c, a plain C99 program that uses the library
    without Python (gcc; links libevl.so and the HIP runtime for hipMalloc / hipMemcpy)."""
    src = os.path.join(ROOT, "tests", "c_abi", "closed_forms.c")
    out = os.path.join(ROOT, "tests", "c_abi", "closed_forms")
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(rocm, "include"), "-I", os.path.join(ROOT, "include"), src, "-o", out,
           "-L", PKG, "-levl", "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-lm",
           "-Wl,-rpath,$ORIGIN/../../paper_2512_10310_amd", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("building the C ABI test program failed:\n" + r.stdout)
    return out


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
