"""The host-side code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only).

Builds a copy of the fp64 oracle (oracle/lg_oracle.c) and a copy of liblonggen_attn.so whose HOST code
(argument checks, the host build of the tile scheduler and cache geometry in csrc/lg_mask.h, launch set-up)
are compiled with -fsanitize=address,undefined, then runs the mask / scheduler / cache pins and the host ABI
checks against those copies in a child process with the sanitizer runtime preloaded.  Any report (out-of-bounds
access, use after free, signed overflow, invalid shift, misaligned access ...) aborts the child."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = "/opt/rocm/lib/llvm/bin/clang"
PINS = ["tests/test_oracle_mask.py", "tests/test_oracle_cache.py", "tests/test_scheduler.py",
        "tests/test_cache_host.py", "tests/test_host_abi.py"]


def asan_runtime():
    found = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    return found[0] if found else None


@pytest.mark.skipif(asan_runtime() is None or not os.path.exists(CLANG), reason="clang sanitizer runtime not found")
def test_pins_pass_with_sanitized_host_code(tmp_path):
    from paper_2410_01485_amd import build as lg_build
    rt = asan_runtime()
    oracle = str(tmp_path / "liblg_oracle_san.so")
    subprocess.check_call([CLANG, "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                           "-shared-libsan", "-O1", "-g", "-shared", "-fPIC", "-std=c11", "-ffp-contract=off",
                           os.path.join(ROOT, "oracle", "lg_oracle.c"), "-o", oracle, "-lm",
                           "-Wl,-rpath,/opt/rocm/lib/llvm/lib"])
    attn = lg_build.build(verbose=False, sanitize_host=True, out=str(tmp_path / "liblonggen_attn_san.so"))
    env = dict(os.environ)
    # the sanitizer runtime must come first among the preloaded libraries; whatever is preloaded already stays
    env["LD_PRELOAD"] = rt + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"     # the interpreter itself is not leak-clean
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["LG_ORACLE_LIB"] = oracle
    env["LONGGEN_ATTN_LIB"] = attn
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"] + PINS,
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    tail = r.stdout[-3000:]
    assert r.returncode == 0, tail
    assert "runtime error" not in r.stdout and "AddressSanitizer" not in r.stdout, tail
    assert " passed" in tail
