"""Build the C-ABI library (hipcc, gfx950 only) in-tree.

    python -m paper_2203_05016_amd.build
    python -m paper_2203_05016_amd.build --host-sanitized   # g++ ASan/UBSan build of the host-only sources

The result is ``paper_2203_05016_amd/libshflbw.so``; it links against the HIP
runtime only (no torch).
"""
import os
import subprocess
import sys
import time

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libshflbw.so")
SOURCES = ["compress.cpp", "pattern_search.cpp", "api_device.hip", "launch_gather_f16.hip", "launch_gather_bf16.hip",
           "layernorm_transpose.hip"]
# packed fp32 instructions are switched off for all device code
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def build(verbose=True, extra=()):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs, procs = [], []
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    t0 = time.time()
    for src in SOURCES:
        obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj] + FLAGS + list(extra)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
        objs.append(obj)
    for src, p in procs:
        out = p.communicate()[0].decode()
        keep = [l for l in out.splitlines() if "packed-fp32-ops" not in l]
        if p.returncode != 0:
            sys.stderr.write(out)
            raise RuntimeError("hipcc failed on %s" % src)
        if verbose and keep:
            print("\n".join(keep))
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call([hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp] + objs)
    os.replace(tmp, LIB)
    if verbose:
        print("built %s in %.1f s" % (LIB, time.time() - t0))
    return LIB


HOST_SOURCES = ["compress.cpp", "pattern_search.cpp"]
HOST_SANITIZED_LIB = os.path.join(HERE, "_build", "libshflbw_host_sanitized.so")


def build_host_sanitized():
    """The host-only part of the library (offline compression, pattern search, the test
    hooks: no HIP call in it) compiled with g++ under AddressSanitizer and
    UndefinedBehaviorSanitizer, as a library of its own for the CPU tests.  Returns
    (path of the library, path of the sanitizer runtime to preload)."""
    os.makedirs(os.path.dirname(HOST_SANITIZED_LIB), exist_ok=True)
    tmp = HOST_SANITIZED_LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                           "-fPIC", "-shared", "-Wall", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                           "-o", tmp] + [os.path.join(CSRC, f) for f in HOST_SOURCES])
    os.replace(tmp, HOST_SANITIZED_LIB)
    runtime = subprocess.check_output(["g++", "-print-file-name=libasan.so"]).decode().strip()
    return HOST_SANITIZED_LIB, os.path.realpath(runtime)


if __name__ == "__main__":
    if sys.argv[1:] == ["--host-sanitized"]:
        print("built %s (preload %s)" % build_host_sanitized())
    else:
        build(extra=sys.argv[1:])
