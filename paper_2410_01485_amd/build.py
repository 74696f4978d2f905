"""Build liblonggen_attn.so from csrc/*.hip with hipcc for gfx950 (cross-compiles without a GPU).

    python -m paper_2410_01485_amd.build
"""
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblonggen_attn.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         # packed-fp32 instructions are kept out of the generated code on purpose
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


# host code (argument checks, host build of the tile scheduler, launch set-up) under AddressSanitizer and
# UndefinedBehaviorSanitizer; the device code is built as usual
SAN_COMPILE = ["-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
               "-Xarch_host", "-fno-sanitize-recover=undefined"]
SAN_LINK = ["-fno-gpu-sanitize", "-fsanitize=address", "-fsanitize=undefined", "-shared-libsan"]


def build(verbose=True, jobs=8, sanitize_host=False, out=None):
    """Compile every translation unit (in parallel) and link the shared library.

    sanitize_host: build a second library (path `out`) whose HOST code runs under ASan + UBSan; a process
    that loads it must have the clang ASan runtime preloaded (tests/test_sanitized_host.py does that)."""
    lib = out or LIB
    objdir = os.path.join(HERE, "_build_san" if sanitize_host else "_build")
    os.makedirs(objdir, exist_ok=True)
    flags = FLAGS + (SAN_COMPILE if sanitize_host else [])
    procs = []
    objs = []
    for src in sources():
        obj = os.path.join(objdir, os.path.basename(src)[:-4] + ".o")
        objs.append(obj)
        cmd = [HIPCC] + flags + ["-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
        while sum(p.poll() is None for _, p in procs) >= jobs:
            procs[0][1].wait()
    failed = False
    for src, p in procs:
        out = p.communicate()[0].decode()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            failed = True
            print("FAILED: %s\n%s" % (src, out), file=sys.stderr)
        elif verbose and out.strip():
            print(out)
    if failed:
        raise RuntimeError("hipcc failed")
    tmp = lib + ".tmp%d" % os.getpid()
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + (SAN_LINK if sanitize_host else []) + ["-o", tmp] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, lib)
    return lib


if __name__ == "__main__":
    print(build())
