"""Builds libdisc.so (host runtime + embedded device header) in-tree with hipcc.

The device kernels themselves are compiled per pattern at registration time through hipRTC
for gfx950; `compile_reference_patterns()` does that for the five benchmark patterns in a
host-only context, so a machine without a GPU can still check that every kernel version
builds.
"""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdisc.so")
SOURCES = ["checker.cpp", "codegen.cpp", "runtime.cpp"]


def _embed_header(build_dir: str) -> str:
    with open(os.path.join(CSRC, "disc_device.h")) as f:
        text = f.read().replace("#pragma once\n", "", 1)   # it becomes the head of the main file
    assert ')DISCHDR"' not in text
    out = os.path.join(build_dir, "device_header_embed.cpp")
    # raw string literals are limited to 64 KiB by some compilers: split in chunks
    chunks = [text[i:i + 12000] for i in range(0, len(text), 12000)]
    body = "\n".join('R"DISCHDR(%s)DISCHDR"' % c for c in chunks)
    with open(out, "w") as f:
        f.write("// generated from disc_device.h -- do not edit\nnamespace disc {\n"
                "extern const char* const kDeviceHeader;\nconst char* const kDeviceHeader =\n%s;\n}\n" % body)
    return out


def build_library(verbose: bool = False) -> str:
    build_dir = os.path.join(HERE, "_build")
    os.makedirs(build_dir, exist_ok=True)
    embed = _embed_header(build_dir)
    # The library holds host code only (checker, code generator, planner, launcher): every
    # device kernel is compiled from disc_device.h + the generated pattern struct through
    # hipRTC with --offload-arch=gfx950, so the host compiler is used here.
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cxx = os.environ.get("CXX", "g++")
    # The one exception: scratch.hip owns a static __device__ array (the scratch memory of
    # disc_launch_static_scratch), so it is compiled as HIP for gfx950 and linked in as an object.
    scratch_obj = os.path.join(build_dir, "scratch.o")
    hipcc = os.path.join(rocm, "bin", "hipcc")
    hcmd = [hipcc, "--offload-arch=gfx950", "-O2", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
            "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c",
            os.path.join(CSRC, "scratch.hip"), "-o", scratch_obj]
    if verbose:
        print(" ".join(hcmd))
    r = subprocess.run(hcmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc compile of scratch.hip failed:\n" + r.stdout + r.stderr)
    cmd = [cxx, "-O2", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wno-unused-result",
           "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(rocm, "include"),
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES] + \
          [embed, scratch_obj, "-L", os.path.join(rocm, "lib"), "-Wl,-rpath," + os.path.join(rocm, "lib"),
           "-lamdhip64", "-lhiprtc"]
    if verbose:
        print(" ".join(cmd))
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("host compile failed:\n" + r.stdout + r.stderr)
    return LIB


def build_sanitized_driver(out_path: str, driver_source: str) -> str:
    """Host code of the library (checker, code generator, planner, launcher) and a C++ driver in ONE
    executable under AddressSanitizer + UndefinedBehaviorSanitizer.  Host code only: device code is
    never built with a sanitizer.  Run it with ASAN_OPTIONS=detect_leaks=0 (the device compiler's
    own library is not instrumented and keeps caches alive)."""
    build_library()                       # (leaves the HIP object of scratch.hip, linked in unsanitized)
    build_dir = os.path.join(HERE, "_build")
    embed = _embed_header(build_dir)
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = [os.environ.get("CXX", "g++"), "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined",
           "-static-libasan", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-DDISC_NO_INTERPOSE",
           "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(rocm, "include"), "-I", os.path.join(ROOT, "include"),
           "-I", CSRC, "-o", out_path, driver_source] + [os.path.join(CSRC, s) for s in SOURCES] + \
          [embed, os.path.join(build_dir, "scratch.o"), "-L", os.path.join(rocm, "lib"),
           "-Wl,-rpath," + os.path.join(rocm, "lib"), "-lamdhip64", "-lhiprtc"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("sanitized host build failed:\n" + r.stdout + r.stderr)
    return out_path


if __name__ == "__main__":
    print(build_library(verbose=True))
