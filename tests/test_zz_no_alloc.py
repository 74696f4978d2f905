"""GPU parity of the allocation-free decode call (lg_sparse_attn_decode_cache_static) through the C ABI:
bit-identical to lg_sparse_attn_decode_cache (same kernels; the partial results of the split over cache
slots go through the library's built-in scratch array instead of a caller's workspace) and within the
decode tolerances of the fp64 oracle, on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest
import torch

import lg_synth
import paper_2410_01485_amd as lg
from gpu_util import DEV, TOL_LSE, TOL_OUT, TOL_REL, assert_close, f32np
from oracle import lg_oracle as O



def one_call(B, Hq, Hkv, N, D, sink, window, block, stride, dtype, seed):
    q, k, v = lg_synth.prefill_inputs(B, Hq, Hkv, N, D, seed, dtype)
    slots = lg.lg_kv_cache_slots(N, sink, window, block, stride)
    kd, vd = k.to(DEV), v.to(DEV)
    # unwritten and dead slots hold values that would wreck the result if they were read
    kc = torch.full((B, Hkv, slots, D), 1.0e4, dtype=dtype, device=DEV)
    vc = torch.full_like(kc, -1.0e4)
    lg.lg_kv_ring_append(kd, vd, kc, vc, 0, sink, window, block, stride)
    q1 = q[:, :, N - 1].contiguous().to(DEV)
    code = lg.LG_BF16 if dtype == torch.bfloat16 else lg.LG_F32
    need = lg.decode_cache_workspace_bytes(B, Hq, Hkv, N, D, sink, window, block, stride, code)
    assert 0 < need <= 8 << 20, "the case must use the split over cache slots, i.e. the scratch"
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    ref_out = torch.full_like(q1, float("nan"))
    ref_lse = torch.full((B, Hq), float("nan"), dtype=torch.float32, device=DEV)
    lg.lg_sparse_attn_decode_cache(q1, kc, vc, ref_out, ref_lse, ws, N, sink, window, block, stride)
    out = torch.full_like(q1, float("nan"))
    lse = torch.full((B, Hq), float("nan"), dtype=torch.float32, device=DEV)
    lg.lg_sparse_attn_decode_cache_static(q1, kc, vc, out, lse, N, sink, window, block, stride)
    torch.cuda.synchronize()
    assert torch.equal(out, ref_out) and torch.equal(lse, ref_lse), "differs from lg_sparse_attn_decode_cache"
    wo, wl = O.fwd(f32np(q), f32np(k), f32np(v), sink, window, block, stride, rows=(N - 1, N))
    tag = "static decode B%d Hq%d Hkv%d N%d s%d w%d b%d st%d %s" % (B, Hq, Hkv, N, sink, window, block, stride, dtype)
    assert_close(f32np(out), wo[:, :, N - 1], TOL_OUT[dtype], TOL_REL[dtype], tag + " out")
    assert_close(f32np(lse), wl[:, :, N - 1], TOL_LSE[dtype], None, tag + " lse")


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_static_scratch_decode_two_calls_second_smaller(dtype):
    # 17 splits of 4160 keys, GQA; then a smaller call (fewer rows, fewer splits, another pattern) that
    # finds the first call's records still in the scratch array
    one_call(2, 8, 2, 6000, 128, 64, 4096, 1, 0, dtype, 301)
    one_call(1, 2, 1, 900, 64, 64, 512, 64, 4, dtype, 302)
    one_call(2, 8, 2, 6000, 128, 64, 4096, 1, 0, dtype, 303)


@pytest.mark.gpu
def test_static_scratch_decode_replays_from_a_graph():
    """The caller the entry point exists for: a decode step captured into a HIP graph (no allocation, no
    clearing node, no synchronisation inside the capture).  The scratch address is looked up at the first
    call on the device, which therefore happens before the capture.  Every replay runs on fresh inputs, with
    eager work between replays, and is compared with the eager workspace call."""
    B, Hq, Hkv, N, D, sink, window, block, stride = 2, 8, 2, 6000, 128, 64, 4096, 1, 0
    dt = torch.bfloat16
    slots = lg.lg_kv_cache_slots(N, sink, window, block, stride)
    kc = torch.zeros(B, Hkv, slots, D, dtype=dt, device=DEV)
    vc = torch.zeros_like(kc)
    q1 = torch.zeros(B, Hq, D, dtype=dt, device=DEV)
    out = torch.empty_like(q1)
    lse = torch.empty(B, Hq, dtype=torch.float32, device=DEV)
    ws = torch.empty(lg.decode_cache_workspace_bytes(B, Hq, Hkv, N, D, sink, window, block, stride, lg.LG_BF16),
                     dtype=torch.uint8, device=DEV)
    ref_out, ref_lse = torch.empty_like(out), torch.empty_like(lse)
    lg.lg_sparse_attn_decode_cache_static(q1, kc, vc, out, lse, N, sink, window, block, stride)   # warm-up
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        lg.lg_sparse_attn_decode_cache_static(q1, kc, vc, out, lse, N, sink, window, block, stride)
    for rep in range(3):
        q, k, v = lg_synth.prefill_inputs(B, Hq, Hkv, N, D, 310 + rep, dt)
        lg.lg_kv_ring_append(k.to(DEV), v.to(DEV), kc, vc, 0, sink, window, block, stride)
        q1.copy_(q[:, :, N - 1])
        out.fill_(float("nan"))
        lse.fill_(float("nan"))
        graph.replay()
        lg.lg_sparse_attn_decode_cache(q1, kc, vc, ref_out, ref_lse, ws, N, sink, window, block, stride)
        torch.cuda.synchronize()
        assert torch.equal(out, ref_out) and torch.equal(lse, ref_lse), rep


def test_static_scratch_limit_and_argument_errors_need_no_gpu():
    # checked before the first HIP call (fake, never dereferenced pointers)
    L, P = lg.lib(), 0x1000

    def call(q=P, B=2, Hq=4, Hkv=2, N=100, D=128, sink=4, window=28, block=1, stride=0, slots=32):
        return L.lg_sparse_attn_decode_cache_static(q, P, P, P, P, B, Hq, Hkv, N, D, sink, window, block, stride,
                                                    slots, lg.LG_BF16, 0.0, None)

    assert call(q=None) == 1 and call(N=0) == 2 and call(Hq=3) == 2 and call(D=32) == 3 and call(slots=31) == 2
    assert call(q=P + 4, N=100000, sink=64, window=4096, slots=4160) == 2          # misaligned, split needed
    # 511 (b, kv head) pairs x 2 splits x 16 query heads per kv head need 8.5 MB of records: refused
    assert lg.decode_cache_workspace_bytes(73, 112, 7, 512, 128, 0, 512, 1, 0, lg.LG_BF16) > 8 << 20
    assert call(B=73, Hq=112, Hkv=7, N=512, sink=0, window=512, slots=512) == 4


def test_scratch_array_is_a_global_symbol_of_the_device_image(tmp_path):
    """hipGetSymbolAddress finds the array by name among the code object's GLOBAL symbols; when the compiler
    keeps a file-scope static device array as a local symbol (an added `used` attribute does that) the HIP
    runtime does not return an error for it but ends the process.  Checked in the generated device code."""
    import os
    import re
    import subprocess
    hipcc = "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    out = tmp_path / "lg_api_device.s"
    subprocess.run([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                    "-packed-fp32-ops", "-S", "--cuda-device-only", "-o", str(out),
                    os.path.join(root, "paper_2410_01485_amd", "csrc", "lg_api.hip")], check=True,
                   capture_output=True, timeout=600)
    text = out.read_text()
    assert re.search(r"^\s*\.globl\s+\S*lg_static_scratch\s*$", text, re.M)
    assert re.search(r"^\s*\.size\s+\S*lg_static_scratch,\s*%d\s*$" % (8 << 20), text, re.M)
