"""Helpers for the GPU parity tests: run an entry point of the C ABI through the Python
binding on seeded inputs and hand the same bytes to the fp64 oracle."""
import numpy as np
import torch

import lg_synth
import paper_2410_01485_amd as lg
from oracle import lg_oracle as O

DEV = "cuda:0"

# Tolerances against the fp64 oracle.
#  bf16 path: outputs are rounded to bf16 (half a unit in the last place = 2^-9 of the value) and P / dS
#  are rounded to bf16 before the second products.  Three bounds, all of which must hold:
#    element, absolute:   |err| <= 2e-2 * max(1, |ref|)                       (the stated tolerance)
#    element, scaled:     |err| <= RMS_K * max(rms(row of ref), rms(ref)) + EL_K * |ref|   (bites when
#                         |ref| << 1: at window 4096 the results have an rms of 0.01 .. 0.03)
#    row (last axis):     ||err_row|| <= ROW_REL * max(||ref_row||, rms(ref) * sqrt(D))
#    tensor:              ||err|| <= 1e-2 * ||ref||
#  RMS_K and ROW_REL are two to three times the largest values measured over the whole GPU suite (bf16:
#  0.036 and 0.012).  dq on the bf16 path gets one more, explicit term: see dq_delta_allowance.
#  float32 path: float32 products and sums over at most a few thousand terms: 1e-4 max-abs.
TOL_OUT = {torch.bfloat16: 2e-2, torch.float32: 1e-4}
TOL_LSE = {torch.bfloat16: 2e-3, torch.float32: 1e-4}
TOL_REL = {torch.bfloat16: 1e-2, torch.float32: 1e-5}
RMS_K = {torch.bfloat16: 8e-2, torch.float32: 1e-4}
EL_K = {torch.bfloat16: 2.0 ** -7, torch.float32: 1e-5}
ROW_REL = {torch.bfloat16: 3e-2, torch.float32: 5e-5}
DELTA_SIGMAS = 6.0   # see dq_delta_allowance


def f32np(t):
    return t.detach().float().cpu().numpy()


def run_fwd(q, k, v, sink, window, block=1, stride=0, scale=0.0, want_lse=True):
    qd, kd, vd = (x.to(DEV) for x in (q, k, v))
    out = torch.full_like(qd, float("nan"))
    lse = torch.full(qd.shape[:3], float("nan"), dtype=torch.float32, device=DEV) if want_lse else None
    lg.lg_sparse_attn_fwd(qd, kd, vd, out, lse, sink, window, block, stride, scale)
    torch.cuda.synchronize()
    return out, lse


def dq_delta_allowance(q, k, g, out_ref, sink, window, block=1, stride=0, scale=None, rows=None):
    """Per-element allowance for dq on the bf16 path (an array like dq).

    The backward receives the forward's output as STORED, i.e. rounded to bf16, and forms
    Delta_i = <dout_i, out_i> from it, while the oracle uses its own fp64 output.  The difference
    delta_i = <dout_i, round(out_i) - out_i> is a sum of D independent rounding errors, each uniform within
    +-2^-9 |dout_id out_id|: standard deviation 2^-9 / sqrt(3) * ||dout_i o out_i||.  It enters
    dS_ij = P_ij (dP_ij - Delta_i) of every key of the row alike, so dq_i is off by
    scale * delta_i * sum_j P_ij k_j.  For rows with thousands of live keys that sum is tiny; for the first
    rows of a sequence (one to a few dozen keys, large P) it is of the size of dq_i itself, so those rows get
    this explicit allowance: DELTA_SIGMAS standard deviations of delta_i times |sum_j P_ij k_j|, the latter
    from the oracle's forward with the keys in the place of the values."""
    kbar, _ = O.fwd(q, k, k, sink, window, block, stride, scale, rows=rows)
    D = q.shape[-1]
    sc = float(scale) if scale is not None and scale > 0 else 1.0 / np.sqrt(D)
    s = np.sqrt(((np.asarray(g, dtype=np.float64) * out_ref) ** 2).sum(-1, keepdims=True))
    return DELTA_SIGMAS * 2.0 ** -9 / np.sqrt(3.0) * s * sc * np.abs(kbar)


def assert_close(got, want, tol, rel=None, what="", by_tensor_max=False, dtype=None, allow=None):
    """Element, row and tensor bounds of the header.  rel = None: the absolute element bound only
    (log-sum-exp values, whose magnitude is of order 10 and whose bound is 2e-3).  dtype: the element type
    of the kernel's result (selects the scaled bounds); taken to be bf16 when tol is the bf16 tolerance.
    allow: per-element allowance added to the scaled element bound and (its row norm) to the row bound."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    assert np.isfinite(got).all(), what + ": non-finite values"
    if not got.size:
        return 0.0
    # element bound: tol for values up to 1 in magnitude, tol * |value| above (a bf16 result of
    # magnitude x carries a rounding step of x * 2^-8 by itself)
    # by_tensor_max (stress inputs with sharply peaked softmax only): the unit is the largest
    # magnitude of the tensor, since each element is a sum of terms of that size that were
    # rounded to bf16 one by one
    err_abs = np.abs(got - want)
    unit = np.abs(want).max() if by_tensor_max else np.abs(want)
    err = (err_abs / np.maximum(1.0, unit)).max()
    assert err <= tol, "%s: max abs err (scaled above 1) %.3e > %.1e" % (what, err, tol)
    if rel is None:
        return err
    if dtype is None:
        dtype = torch.bfloat16 if tol >= 1e-3 else torch.float32
    # relative to the reference's norm, floored at an rms of 1e-3 so that results that are
    # (nearly) zero by construction are judged by the absolute bound alone
    rms = max(np.sqrt(np.mean(want * want)), 1e-3)
    r = np.linalg.norm(got - want) / (rms * np.sqrt(got.size))
    assert r <= rel, "%s: rel l2 err %.3e > %.1e" % (what, r, rel)
    # scaled element bound: a wrong element in a tensor of small values cannot hide under the absolute bound
    # (errors of an element grow with the terms that were summed into its ROW -- the first keys of a
    # sequence collect gradient from every query and are far larger than the tensor's rms --, so the unit
    # is the larger of the row's and the tensor's rms)
    el_unit = np.abs(want).max() if by_tensor_max else np.abs(want)
    row_rms = np.sqrt(np.mean(want * want, axis=-1, keepdims=True)) if got.ndim >= 2 else rms
    bound = RMS_K[dtype] * np.maximum(row_rms, rms) + EL_K[dtype] * el_unit
    if allow is not None:
        bound = bound + allow
    worst = (err_abs / bound).max()
    assert worst <= 1.0, "%s: element err %.3e at %s exceeds %.1e * rms (%.3e) + %.1e * |ref|" % (
        what, err_abs.flat[np.argmax(err_abs / bound)], np.unravel_index(np.argmax(err_abs / bound), got.shape),
        RMS_K[dtype], rms, EL_K[dtype])
    # row bound (rows = vectors along the last axis): a wrong row cannot hide in the tensor's norm
    if got.ndim >= 2 and got.shape[-1] > 1:
        en = np.linalg.norm(got - want, axis=-1)
        rn = np.maximum(np.linalg.norm(want, axis=-1), rms * np.sqrt(got.shape[-1]))
        if by_tensor_max:
            rn = np.full_like(rn, max(rn.max(), np.abs(want).max() * np.sqrt(got.shape[-1])))
        if allow is not None:
            en = np.maximum(en - np.linalg.norm(np.broadcast_to(allow, got.shape), axis=-1), 0.0)
        rr = (en / rn).max()
        assert rr <= ROW_REL[dtype], "%s: row %s rel l2 err %.3e > %.1e" % (
            what, np.unravel_index(np.argmax(en / rn), en.shape), rr, ROW_REL[dtype])
    return err


def check_fwd(B, Hq, Hkv, N, D, sink, window, block=1, stride=0, dtype=torch.bfloat16, seed=1, q_mul=1.0,
              scale=0.0):
    q, k, v = lg_synth.prefill_inputs(B, Hq, Hkv, N, D, seed, dtype, q_mul=q_mul)
    out, lse = run_fwd(q, k, v, sink, window, block, stride, scale)
    wo, wl = O.fwd(f32np(q), f32np(k), f32np(v), sink, window, block, stride, scale if scale > 0 else None)
    tag = "fwd B%d Hq%d Hkv%d N%d D%d s%d w%d b%d st%d %s" % (B, Hq, Hkv, N, D, sink, window, block, stride, dtype)
    assert_close(f32np(out), wo, TOL_OUT[dtype], TOL_REL[dtype], tag + " out")
    assert_close(f32np(lse), wl, TOL_LSE[dtype], None, tag + " lse")
