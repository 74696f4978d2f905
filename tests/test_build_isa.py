"""Generated-code checks for the kernels that name AGPR blocks directly.

The 64-keys-per-wave dk/dv kernel keeps its 16 accumulators in fixed AGPR blocks that only its own
inline matrix instructions touch.  That is only sound while the compiler itself puts nothing into
AGPRs in that kernel and spills nothing; this test compiles the file to assembly (no GPU needed) and
checks exactly that.
"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2410_01485_amd", "csrc", "lg_bwd_bf16.hip")


def _hipcc():
    for c in ("/opt/rocm/bin/hipcc", shutil.which("hipcc")):
        if c and os.path.exists(c):
            return c
    return None


@pytest.fixture(scope="module")
def wide_kernels(tmp_path_factory):
    hipcc = _hipcc()
    if hipcc is None:
        pytest.skip("hipcc not available")
    out = tmp_path_factory.mktemp("isa") / "lg_bwd_bf16.s"
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-S", "--cuda-device-only", "-o", str(out), SRC]
    subprocess.run(cmd, check=True, capture_output=True, timeout=600)
    text = out.read_text()
    kernels = {}
    for mt in re.finditer(r"^(_ZN\S*dkdv_wide_bf16_kernel\S*):.*?^\.Lfunc_end\d+:", text, re.S | re.M):
        kernels[mt.group(1)] = mt.group(0)
    meta = {}   # kernel name -> its entry in the code object metadata (one "- .agpr_count: ..." block each)
    for entry in re.split(r"\n  - (?=\.agpr_count:)", text):
        mt = re.search(r"\.name:\s+(_ZN\S*dkdv_wide_bf16_kernel\S*)", entry)
        if mt and entry.startswith(".agpr_count"):
            meta[mt.group(1)] = entry
    return kernels, meta, text


def test_wide_dkdv_instances_present(wide_kernels):
    kernels, meta, _ = wide_kernels
    assert len(kernels) == 2, sorted(kernels)          # TOKEN = true / false


def test_compiler_keeps_out_of_the_agprs(wide_kernels):
    kernels, _, _ = wide_kernels
    for name, body in kernels.items():
        # nothing but the kernel's own statements may write an AGPR: they do so only as the
        # destination of matrix instructions
        assert "v_accvgpr_write" not in body, name
        assert "v_accvgpr_mov" not in body, name
        # the copy-out reads each of the 256 accumulator registers exactly once
        reads = re.findall(r"v_accvgpr_read_b32\s+v\d+,\s*a(\d+)", body)
        assert sorted(int(r) for r in reads) == list(range(256)), name
        # AGPRs appear otherwise only as matrix accumulators (destination == addend)
        for line in body.splitlines():
            line = line.split(";")[0]
            if "a[" in line and "v_mfma" in line:
                ops = [o.strip() for o in line.split(None, 1)[1].split(",")]
                if ops[0].startswith("a["):
                    assert ops[3] in (ops[0], "0"), line
            elif re.search(r"\ba\[\d+:\d+\]|\ba\d+\b", line) and "v_accvgpr_read" not in line:
                raise AssertionError(f"{name}: AGPR used outside the accumulators: {line.strip()}")


def test_no_spills_in_wide_dkdv(wide_kernels):
    kernels, meta, _ = wide_kernels
    for name, body in kernels.items():
        assert "scratch_" not in body, name
    assert len(meta) == 2
    for name, md in meta.items():
        assert re.search(r"\.private_segment_fixed_size:\s+0\b", md), name
        assert re.search(r"\.vgpr_spill_count:\s+0\b", md), name
        assert re.search(r"\.agpr_count:\s+256\b", md), name
