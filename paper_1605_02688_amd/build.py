"""Builds libewf.so (host library + ahead-of-time auxiliary kernels for gfx950) in-tree.

    python -m paper_1605_02688_amd.build

With ``--sanitize`` it builds libewf_asan.so instead: the host code (everything but the kernels)
under AddressSanitizer and UndefinedBehaviorSanitizer.  The host-only tests then run as

    python -m paper_1605_02688_amd.build --sanitize
    EWF_LIBRARY=$PWD/paper_1605_02688_amd/libewf_asan.so \
        LD_PRELOAD="$(gcc -print-file-name=libasan.so) $(gcc -print-file-name=libubsan.so)" \
        ASAN_OPTIONS=detect_leaks=0 python -m pytest tests -m "not gpu" -q

The kernel prelude (csrc/kernels/ewf_prelude.hip.h) is embedded into the library as a
string so that the run-time compiler can see it on machines without the source tree.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libewf.so")
BUILD_DIR = os.path.join(HERE, "_build")

HOST_SOURCES = ["ewf_ir.cpp", "ewf_rewrite.cpp", "ewf_grad.cpp", "ewf_canon.cpp", "ewf_codegen.cpp", "ewf_gen_tile.cpp", "ewf_gen_row.cpp", "ewf_gen_col.cpp", "ewf_gen_lane.cpp", "ewf_rtc.cpp", "ewf_multi.cpp", "ewf_api.cpp"]
HIP_SOURCES = ["ewf_aux.hip"]
# packed-fp32 instructions stay off in all device code of this library
HIP_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _embed_prelude() -> None:
    src = os.path.join(CSRC, "kernels", "ewf_prelude.hip.h")
    text = open(src).read()
    delim = "EWFPRELUDE"
    assert ")" + delim not in text
    # string literals have a length limit in some compilers; split into chunks
    chunks = [text[i:i + 8000] for i in range(0, len(text), 8000)]
    with open(os.path.join(BUILD_DIR, "ewf_prelude_embed.inc"), "w") as f:
        for c in chunks:
            f.write(f'R"{delim}({c}){delim}"\n')


def build(verbose: bool = False, sanitize: bool = False) -> str:
    os.makedirs(BUILD_DIR, exist_ok=True)
    _embed_prelude()
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    common = ["-O2", "-fPIC", "-std=c++17", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-I", BUILD_DIR,
              "-Wall", "-Wno-unused-result"]
    san = ["-fsanitize=address,undefined", "-fno-omit-frame-pointer", "-g"] if sanitize else []
    procs = []
    for s in HOST_SOURCES + HIP_SOURCES:
        obj = os.path.join(BUILD_DIR, s + (".asan.o" if sanitize else ".o"))
        if s.endswith(".hip"):      # (device code is never instrumented: host side only)
            cmd = [hipcc, "-c", os.path.join(CSRC, s), "-o", obj] + common + HIP_FLAGS
        else:       # plain C++: no device code in the host sources
            cmd = ["g++", "-c", os.path.join(CSRC, s), "-o", obj, "-D__HIP_PLATFORM_AMD__",
                   "-I", "/opt/rocm/include"] + common + san
        if verbose:
            print(" ".join(cmd))
        procs.append((s, subprocess.Popen(cmd)))
        objs.append(obj)
    for s, p in procs:
        if p.wait() != 0:
            raise RuntimeError(f"compiling {s} failed")
    lib = os.path.join(HERE, "libewf_asan.so") if sanitize else LIB
    tmp = lib + f".tmp{os.getpid()}"
    cmd = [hipcc, "-shared", "-o", tmp] + objs + ["-lhiprtc", "--offload-arch=gfx950"]
    if sanitize:    # the sanitizer's run-time library comes from the process (LD_PRELOAD), as for any instrumented plug-in
        cmd += ["-Wl,--allow-shlib-undefined"]
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    os.replace(tmp, lib)
    if sanitize:
        return lib
    # the plain C program that drives the library through its C ABI (used by a GPU test)
    csrc = os.path.join(ROOT, "tests", "c_abi", "c1_from_c.c")
    if os.path.exists(csrc):
        cmd = ["gcc", csrc, "-o", os.path.join(ROOT, "tests", "c_abi", "c1_from_c"), "-O2", "-std=c11", "-Wall",
               "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROOT, "include"), "-I", "/opt/rocm/include",
               "-L", HERE, "-lewf", "-L", "/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath," + HERE, "-Wl,-rpath,/opt/rocm/lib"]
        if verbose:
            print(" ".join(cmd))
        subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv, sanitize="--sanitize" in sys.argv))
