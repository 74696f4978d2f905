"""Generated-code checks for the kernels that name AGPR blocks directly.

The 64-keys-per-wave dk/dv kernel and the 64-rows-per-wave dq kernel keep their accumulators (and
the dq kernel its Q / dO fragments) in fixed AGPR blocks that only their own inline statements
touch.  That is only sound while the compiler itself puts nothing into AGPRs in those kernels and
spills nothing; this test compiles the file to assembly (no GPU needed) and checks exactly that.
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
    for mt in re.finditer(r"^(_ZN\S*(?:dkdv|dq)_wide_bf16_kernel\S*):.*?^\.Lfunc_end\d+:", text, re.S | re.M):
        kernels[mt.group(1)] = mt.group(0)
    meta = {}   # kernel name -> its entry in the code object metadata (one "- .agpr_count: ..." block each)
    for entry in re.split(r"\n  - (?=\.agpr_count:)", text):
        mt = re.search(r"\.name:\s+(_ZN\S*(?:dkdv|dq)_wide_bf16_kernel\S*)", entry)
        if mt and entry.startswith(".agpr_count"):
            meta[mt.group(1)] = entry
    return kernels, meta, text


def test_wide_instances_present(wide_kernels):
    kernels, meta, text = wide_kernels
    # the global->LDS copies name their base address as a scalar operand; a base the compiler had
    # computed with vector instructions showed up as a vector register pair there, which does not assemble
    assert not re.search(r"global_load_lds_dwordx4\s+v\d+,\s*v\[", text)
    assert len(kernels) == 5, sorted(kernels)          # dq: TOKEN = true / false; dk/dv: those two and the column instance


def test_compiler_keeps_out_of_the_agprs(wide_kernels):
    kernels, _, _ = wide_kernels
    for name, body in kernels.items():
        is_dq = "dq_wide" in name
        nacc = 128 if is_dq else 256      # accumulator registers a0 .. a(nacc-1)
        # the only AGPR writes besides matrix results: the dq kernel stores its 32 fragments once
        writes = re.findall(r"v_accvgpr_write_b32\s+a(\d+),", body)
        assert sorted(int(r) for r in writes) == (list(range(128, 256)) if is_dq else []), name
        assert "v_accvgpr_mov" not in body, name
        # the copy-out reads each accumulator register exactly once
        reads = re.findall(r"v_accvgpr_read_b32\s+v\d+,\s*a(\d+)", body)
        assert sorted(int(r) for r in reads) == list(range(nacc)), name
        # otherwise AGPRs appear only in matrix instructions: as accumulator (destination == addend,
        # inside the accumulator range) or, in the dq kernel, as the second operand (a fragment)
        for line in body.splitlines():
            line = line.split(";")[0]
            if "v_mfma" in line:
                ops = [o.strip() for o in line.split(None, 1)[1].split(",")]
                if ops[0].startswith("a["):
                    assert ops[3] in (ops[0], "0"), line
                    assert int(re.match(r"a\[(\d+):", ops[0]).group(1)) < nacc, line
                else:
                    assert not ops[3].startswith("a["), line
                assert not ops[1].startswith("a["), line
                if ops[2].startswith("a["):
                    assert is_dq and int(re.match(r"a\[(\d+):", ops[2]).group(1)) >= 128, line
            elif re.search(r"\ba\[\d+:\d+\]|\ba\d+\b", line) and "v_accvgpr_" not in line:
                raise AssertionError(f"{name}: AGPR used outside the kernel's own statements: {line.strip()}")


def test_no_spills_in_wide_kernels(wide_kernels):
    kernels, meta, _ = wide_kernels
    for name, body in kernels.items():
        assert "scratch_" not in body, name
    assert len(meta) == 5
    for name, md in meta.items():
        assert re.search(r"\.private_segment_fixed_size:\s+0\b", md), name
        assert re.search(r"\.vgpr_spill_count:\s+0\b", md), name
        assert re.search(r"\.agpr_count:\s+256\b", md), name


def _regs(op):
    """VGPR numbers named by one operand (v12, v[4:7]); AGPRs and everything else: none."""
    mt = re.match(r"v\[(\d+):(\d+)\]$", op)
    if mt:
        return set(range(int(mt.group(1)), int(mt.group(2)) + 1))
    mt = re.match(r"v(\d+)$", op)
    return {int(mt.group(1))} if mt else set()


def test_matrix_operands_are_not_written_just_before_use(wide_kernels):
    """An inline matrix instruction that read a register right after a vector instruction wrote it
    got stale lanes (the compiler spaces its own instructions, not inline ones).  The kernels keep
    every such write at least one matrix instruction (or a long s_nop) ahead; check the generated
    code: between a matrix instruction and the previous one (or the previous s_nop of 8+ slots),
    no vector instruction may write one of its VGPR operands."""
    kernels, _, _ = wide_kernels
    for name, body in kernels.items():
        written = {}          # VGPR -> text of the vector instruction that wrote it since the last fence
        for raw in body.splitlines():
            line = raw.split(";")[0].strip()
            if not line or line.startswith(".") or line.endswith(":"):
                if line.endswith(":"):
                    written = dict(written)   # labels: keep (conservative: straight-line and joins alike)
                continue
            op = line.split()[0]
            ops = [o.strip() for o in line.split(None, 1)[1].split(",")] if " " in line else []
            if op.startswith("v_mfma"):
                for src in ops[1:4]:
                    hit = _regs(src) & set(written)
                    assert not hit, f"{name}: {line}  reads v{min(hit)} written by: {written[min(hit)]}"
                written = {}
            elif op == "s_nop" and ops and int(ops[0]) >= 7:
                written = {}
            elif op.startswith(("ds_read", "global_load", "buffer_load", "scratch_load")) and "lds" not in op:
                for r in _regs(ops[0]) if ops else ():   # reloaded from memory: waited for by counter
                    written.pop(r, None)
            elif op.startswith("v_") and not op.startswith("v_accvgpr_write") and not op.startswith("v_cmp"):
                for r in _regs(ops[0]) if ops else ():
                    written[r] = line
                if op.startswith("v_permlane32_swap") and len(ops) > 1:
                    for r in _regs(ops[1]):
                        written[r] = line


MFMA_GAP = 4       # matrix instructions that must lie between an inline matrix instruction and a reader of its result
NOP_STATES = 11    # ... or this many idle issue slots (what an 8-pass matrix instruction needs before a vector access)


def _all_regs(text):
    """Every VGPR / AGPR a piece of operand text names: ('v', n) / ('a', n)."""
    regs = set()
    for kind, lo, hi in re.findall(r"\b([va])\[(\d+):(\d+)\]", text):
        regs |= {(kind, r) for r in range(int(lo), int(hi) + 1)}
    for kind, n in re.findall(r"\b([va])(\d+)\b", text):
        regs.add((kind, int(n)))
    return regs


def test_matrix_results_are_not_touched_too_early(wide_kernels):
    """The other direction of the hazard: a vector or memory instruction that reads (or overwrites) a register
    an inline matrix instruction wrote must come at least MFMA_GAP matrix instructions (or NOP_STATES idle
    slots) later; the hardware does not wait for it and the compiler does not see inside the statement.  The
    kernels place such readers six matrix instructions after the last one of an accumulation chain; this checks
    the generated code (straight-line order, which is how the unrolled steps run).  A matrix instruction that
    continues a chain on the same destination is exempt (the pipe forwards its own accumulator)."""
    kernels, _, _ = wide_kernels
    for name, body in kernels.items():
        written = {}              # register -> (matrix instructions issued, idle slots) when a matrix instruction wrote it
        n_mfma = n_nop = 0
        for raw in body.splitlines():
            line = raw.split(";")[0].strip()
            if not line or line.startswith(".") or line.endswith(":"):
                continue
            op = line.split()[0]
            rest = line.split(None, 1)[1] if " " in line else ""
            if op.startswith("v_mfma"):
                ops = [o.strip() for o in rest.split(",")]
                dst = _all_regs(ops[0])
                for r in (_all_regs(ops[1]) | _all_regs(ops[2])) & set(written):   # results are never fed back as A / B
                    raise AssertionError(f"{name}: {line} reads {r} written by a matrix instruction")
                if _all_regs(ops[3]) != dst:                                        # not a chain on its own accumulator
                    for r in _all_regs(ops[3]) & set(written):
                        w = written[r]
                        assert n_mfma - w[0] >= MFMA_GAP or n_nop - w[1] >= NOP_STATES, f"{name}: {line} (addend {r})"
                n_mfma += 1
                for r in dst:
                    written[r] = (n_mfma, n_nop)
            elif op == "s_nop":
                n_nop += int(rest.strip()) + 1
            elif op.startswith(("v_", "ds_", "global_", "buffer_", "scratch_", "flat_")):
                for r in _all_regs(rest) & set(written):
                    w = written.pop(r)
                    assert n_mfma - w[0] >= MFMA_GAP or n_nop - w[1] >= NOP_STATES, \
                        f"{name}: {line} touches {r} {n_mfma - w[0]} matrix instructions after it was written"
