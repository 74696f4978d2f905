"""Helpers for the GPU parity tests: run an entry point of the C ABI through the Python
binding on seeded inputs and hand the same bytes to the fp64 oracle."""
import numpy as np
import torch

import lg_synth
import paper_2410_01485_amd as lg
from oracle import lg_oracle as O

DEV = "cuda:0"

# Tolerances against the fp64 oracle.
#  bf16 path: outputs are rounded to bf16 (relative step 2^-8 = 3.9e-3) and P is rounded to bf16
#  before the second product; with |out| of order 1 the error stays below 2e-2 max-abs.
#  float32 path: float32 products and sums over at most a few thousand terms: 1e-4 max-abs.
TOL_OUT = {torch.bfloat16: 2e-2, torch.float32: 1e-4}
TOL_LSE = {torch.bfloat16: 2e-3, torch.float32: 1e-4}
TOL_REL = {torch.bfloat16: 1e-2, torch.float32: 1e-5}


def f32np(t):
    return t.detach().float().cpu().numpy()


def run_fwd(q, k, v, sink, window, block=1, stride=0, scale=0.0, want_lse=True):
    qd, kd, vd = (x.to(DEV) for x in (q, k, v))
    out = torch.full_like(qd, float("nan"))
    lse = torch.full(qd.shape[:3], float("nan"), dtype=torch.float32, device=DEV) if want_lse else None
    lg.lg_sparse_attn_fwd(qd, kd, vd, out, lse, sink, window, block, stride, scale)
    torch.cuda.synchronize()
    return out, lse


def assert_close(got, want, tol, rel=None, what="", by_tensor_max=False):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    assert np.isfinite(got).all(), what + ": non-finite values"
    # element bound: tol for values up to 1 in magnitude, tol * |value| above (a bf16 result of
    # magnitude x carries a rounding step of x * 2^-8 by itself)
    # by_tensor_max (stress inputs with sharply peaked softmax only): the unit is the largest
    # magnitude of the tensor, since each element is a sum of terms of that size that were
    # rounded to bf16 one by one
    unit = np.abs(want).max() if (by_tensor_max and got.size) else np.abs(want)
    excess = np.abs(got - want) / np.maximum(1.0, unit)
    err = excess.max() if got.size else 0.0
    assert err <= tol, "%s: max abs err (scaled above 1) %.3e > %.1e" % (what, err, tol)
    if rel is not None and got.size:
        # relative to the reference's norm, floored at an rms of 1e-3 so that results that are
        # (nearly) zero by construction are judged by the absolute bound alone
        r = np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-3 * np.sqrt(got.size))
        assert r <= rel, "%s: rel l2 err %.3e > %.1e" % (what, r, rel)
    return err


def check_fwd(B, Hq, Hkv, N, D, sink, window, block=1, stride=0, dtype=torch.bfloat16, seed=1, q_mul=1.0,
              scale=0.0):
    q, k, v = lg_synth.prefill_inputs(B, Hq, Hkv, N, D, seed, dtype, q_mul=q_mul)
    out, lse = run_fwd(q, k, v, sink, window, block, stride, scale)
    wo, wl = O.fwd(f32np(q), f32np(k), f32np(v), sink, window, block, stride, scale if scale > 0 else None)
    tag = "fwd B%d Hq%d Hkv%d N%d D%d s%d w%d b%d st%d %s" % (B, Hq, Hkv, N, D, sink, window, block, stride, dtype)
    assert_close(f32np(out), wo, TOL_OUT[dtype], TOL_REL[dtype], tag + " out")
    assert_close(f32np(lse), wl, TOL_LSE[dtype], None, tag + " lse")
