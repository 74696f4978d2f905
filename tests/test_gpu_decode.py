"""GPU parity: lg_sparse_attn_decode (through the C ABI) against the fp64 oracle."""
import numpy as np
import pytest
import torch

import lg_synth
import paper_2410_01485_amd as lg
from gpu_util import DEV, TOL_LSE, TOL_OUT, TOL_REL, assert_close, f32np
from oracle import lg_oracle as O

pytestmark = pytest.mark.gpu


def run_decode(q, kc, vc, N, sink, window, scale=0.0):
    qd, kd, vd = (x.to(DEV) for x in (q, kc, vc))
    B, Hq, D = q.shape
    Hkv = kc.shape[1]
    code = lg.LG_BF16 if q.dtype == torch.bfloat16 else lg.LG_F32
    need = lg.decode_workspace_bytes(B, Hq, Hkv, N, D, sink, window, code)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=DEV)
    out = torch.full_like(qd, float("nan"))
    lse = torch.full((B, Hq), float("nan"), dtype=torch.float32, device=DEV)
    lg.lg_sparse_attn_decode(qd, kd, vd, out, lse, ws, N, sink, window, 1, 0, scale)
    torch.cuda.synchronize()
    return out, lse


def check_decode(B, Hq, Hkv, D, sink, window, N, dtype, seed):
    q, kc, vc = lg_synth.decode_inputs(B, Hq, Hkv, sink + window, D, seed, dtype)
    valid = min(N, sink + window)
    # slots that are not valid yet hold garbage that must never be read into the result
    kc[:, :, valid:] = 1.0e4
    vc[:, :, valid:] = -1.0e4
    out, lse = run_decode(q, kc, vc, N, sink, window)
    wo, wl = O.decode(f32np(q), f32np(kc), f32np(vc), N, sink, window)
    tag = "decode B%d Hq%d Hkv%d D%d s%d w%d N%d %s" % (B, Hq, Hkv, D, sink, window, N, dtype)
    assert_close(f32np(out), wo, TOL_OUT[dtype], TOL_REL[dtype], tag + " out")
    assert_close(f32np(lse), wl, TOL_LSE[dtype], None, tag + " lse")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (8, 4), (8, 2), (8, 1), (6, 2), (16, 1)])
def test_decode_groups(dtype, D, Hq, Hkv):
    check_decode(2, Hq, Hkv, D, 4, 300, 5000, dtype, seed=11)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("N", [1, 2, 63, 64, 65, 303, 304, 305, 100000])
def test_decode_partial_fill_and_sizes(dtype, N):
    check_decode(1, 2, 2, 128, 4, 300, N, dtype, seed=12)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_decode_split_and_single_pass(dtype):
    check_decode(1, 1, 1, 128, 64, 4096, 131072, dtype, seed=13)    # few rows: split over workgroups
    check_decode(40, 32, 32, 128, 16, 240, 7000, dtype, seed=14)    # many rows: one workgroup each


def test_decode_equals_last_row_of_prefill():
    # the ring cache built from a longer context by the slot map reproduces row N-1 of the forward
    B, Hq, Hkv, D, sink, window, N = 1, 4, 2, 128, 8, 120, 1000
    q, k, v = lg_synth.prefill_inputs(B, Hq, Hkv, N, D, 15, torch.bfloat16)
    kc, vc = O.build_ring_cache(k.float().numpy(), v.float().numpy(), sink, window)
    kc, vc = torch.as_tensor(kc).to(torch.bfloat16), torch.as_tensor(vc).to(torch.bfloat16)
    out, lse = run_decode(q[:, :, N - 1].contiguous(), kc, vc, N, sink, window)
    wo, wl = O.fwd(f32np(q), f32np(k), f32np(v), sink, window, rows=(N - 1, N))
    assert_close(f32np(out), wo[:, :, N - 1], TOL_OUT[torch.bfloat16], TOL_REL[torch.bfloat16], "decode vs prefill row")
    assert_close(f32np(lse), wl[:, :, N - 1], TOL_LSE[torch.bfloat16], None, "decode vs prefill lse")


def test_config5_full_size():
    # B16, 32 heads, D128, ring of 64 sink + 4096 window slots from a 131072-token context
    B, H, D, sink, window, N = 16, 32, 128, 64, 4096, 131072
    q, kc, vc = lg_synth.decode_inputs(B, H, H, sink + window, D, 20241006, torch.bfloat16, device=DEV)
    need = lg.decode_workspace_bytes(B, H, H, N, D, sink, window, lg.LG_BF16)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=DEV)
    out = torch.empty_like(q)
    lse = torch.empty(B, H, dtype=torch.float32, device=DEV)
    lg.lg_sparse_attn_decode(q, kc, vc, out, lse, ws, N, sink, window)
    torch.cuda.synchronize()
    for b in (0, 7, 15):      # the oracle recomputes three whole sequences
        wo, wl = O.decode(f32np(q[b:b + 1]), f32np(kc[b:b + 1]), f32np(vc[b:b + 1]), N, sink, window)
        assert_close(f32np(out[b:b + 1]), wo, TOL_OUT[torch.bfloat16], TOL_REL[torch.bfloat16], "cfg5 out b%d" % b)
        assert_close(f32np(lse[b:b + 1]), wl, TOL_LSE[torch.bfloat16], None, "cfg5 lse b%d" % b)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("D,Hq,Hkv,N", [(128, 4, 4, 5000), (64, 8, 2, 5000), (128, 2, 1, 37), (128, 3, 3, 1)])
def test_split_over_head_dim_variant_matches_oracle(dtype, D, Hq, Hkv, N):
    # the measurement aid that splits the head dimension (the paper's decode design) computes the same thing
    B, sink, window = 2, 4, 300
    q, kc, vc = lg_synth.decode_inputs(B, Hq, Hkv, sink + window, D, 17, dtype)
    valid = min(N, sink + window)
    kc[:, :, valid:] = 1.0e4
    vc[:, :, valid:] = -1.0e4
    qd, kd, vd = (x.to(DEV) for x in (q, kc, vc))
    out = torch.full_like(qd, float("nan"))
    lse = torch.full((B, Hq), float("nan"), dtype=torch.float32, device=DEV)
    lg.lg_debug_decode_split_headdim(qd, kd, vd, out, lse, N, sink, window)
    torch.cuda.synchronize()
    wo, wl = O.decode(f32np(q), f32np(kc), f32np(vc), N, sink, window)
    assert_close(f32np(out), wo, TOL_OUT[dtype], TOL_REL[dtype], "split-D decode out")
    assert_close(f32np(lse), wl, TOL_LSE[dtype], None, "split-D decode lse")
