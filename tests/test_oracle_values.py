"""Pins for the oracle's forward, backward and decode values.

Nothing here calls the HIP path.  Checks: library attention (torch CPU fp64
scaled_dot_product_attention and autograd) driven by the hand-written mask fixtures;
plain causal attention when the window covers everything; closed forms (zero queries,
needle keys); softmax invariants; finite differences; GQA by explicit repetition.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import lg_synth
from conftest import GOLDEN_MASKS, load_golden_mask
from oracle import lg_oracle as O


def inputs(B, Hq, Hkv, N, D, seed, with_dout=False, q_mul=1.0):
    t = lg_synth.prefill_inputs(B, Hq, Hkv, N, D, seed, torch.float32, with_dout, q_mul)
    return [x.numpy() for x in t]


def sdpa(q, k, v, mask=None, causal=False, scale=None):
    """torch's library attention in fp64 on the CPU; K/V repeated for GQA."""
    q, k, v = (torch.as_tensor(np.asarray(x, dtype=np.float64)) for x in (q, k, v))
    G = q.shape[1] // k.shape[1]
    k = k.repeat_interleave(G, dim=1)
    v = v.repeat_interleave(G, dim=1)
    am = None if mask is None else torch.as_tensor(mask.astype(bool))
    return F.scaled_dot_product_attention(q, k, v, attn_mask=am, is_causal=causal, scale=scale)


def token_mask(N, sink, window):
    i = np.arange(N)[:, None]
    j = np.arange(N)[None, :]
    return (j <= i) & ((j < sink) | (i - j < window))


@pytest.mark.parametrize("name", GOLDEN_MASKS)
def test_fwd_matches_library_attention_on_hand_written_masks(name):
    p, m = load_golden_mask(name)
    q, k, v = inputs(2, 4, 2, p["N"], 8, seed=11)
    out, lse = O.fwd(q, k, v, p["sink"], p["window"], p["block"], p["stride"])
    want = sdpa(q, k, v, mask=m).numpy()
    assert np.abs(out - want).max() < 1e-12
    # lse against a direct logsumexp over the fixture's live keys
    kk = np.repeat(k, 2, axis=1).astype(np.float64)
    s = np.einsum("bhid,bhjd->bhij", q.astype(np.float64), kk) / np.sqrt(8)
    s = np.where(m.astype(bool), s, -np.inf)
    assert np.abs(lse - torch.logsumexp(torch.as_tensor(s), dim=-1).numpy()).max() < 1e-12


def test_fwd_config1_shape_matches_dense_masked_attention():
    # N=1024, D=64, sink=16, window=128: the small benchmark configuration
    q, k, v = inputs(1, 1, 1, 1024, 64, seed=20241002)
    out, lse = O.fwd(q, k, v, 16, 128)
    want = sdpa(q, k, v, mask=token_mask(1024, 16, 128)).numpy()
    assert np.abs(out - want).max() < 1e-11


@pytest.mark.parametrize("kw", [dict(sink=0, window=300), dict(sink=7, window=256),
                                dict(sink=0, window=8, block=8, stride=1)])
def test_fwd_reduces_to_causal_attention(kw):
    q, k, v = inputs(1, 4, 2, 200, 64, seed=5)
    out, _ = O.fwd(q, k, v, **kw)
    want = sdpa(q, k, v, causal=True).numpy()
    assert np.abs(out - want).max() < 1e-12


def test_fwd_custom_scale_and_pure_sliding_window():
    q, k, v = inputs(1, 2, 2, 64, 16, seed=6)
    out, _ = O.fwd(q, k, v, 0, 5, scale=0.37)
    want = sdpa(q, k, v, mask=token_mask(64, 0, 5), scale=0.37).numpy()
    assert np.abs(out - want).max() < 1e-12


@pytest.mark.parametrize("name", GOLDEN_MASKS)
def test_zero_queries_give_uniform_average_closed_form(name):
    p, m = load_golden_mask(name)
    _, k, v = inputs(1, 2, 1, p["N"], 8, seed=3)
    q = np.zeros((1, 2, p["N"], 8), np.float32)
    out, lse = O.fwd(q, k, v, p["sink"], p["window"], p["block"], p["stride"])
    cnt = m.sum(1).astype(np.float64)
    assert np.abs(lse - np.log(cnt)[None, None]).max() < 1e-14
    mean_v = (m.astype(np.float64) @ v[0, 0].astype(np.float64)) / cnt[:, None]
    assert np.abs(out[0, 0] - mean_v).max() < 1e-14
    assert np.abs(out[0, 1] - mean_v).max() < 1e-14


def test_needle_key_is_retrieved_iff_live():
    p, m = load_golden_mask("mask_block_strided.txt")
    N, D = p["N"], 8
    rng = np.random.default_rng(0)
    v = rng.standard_normal((1, 1, N, D)).astype(np.float32)
    for needle in (0, 3, 4, 7, 10):
        k = np.zeros((1, 1, N, D), np.float32)
        k[0, 0, needle, 0] = 400.0
        q = np.zeros((1, 1, N, D), np.float32)
        q[..., 0] = 1.0
        out, _ = O.fwd(q, k, v, p["sink"], p["window"], p["block"], p["stride"])
        for i in range(N):
            hit = np.abs(out[0, 0, i] - v[0, 0, needle]).max() < 1e-9
            assert hit == bool(m[i, needle])


def test_softmax_invariants():
    p, m = load_golden_mask("mask_sink_window_token.txt")
    N, D = p["N"], 8
    q, k, v = inputs(1, 1, 1, N, D, seed=9)
    out, lse = O.fwd(q, k, v, p["sink"], p["window"])
    # probabilities rebuilt from lse sum to one over the live keys, and rebuild out
    s = (q[0, 0].astype(np.float64) @ k[0, 0].astype(np.float64).T) / np.sqrt(D)
    P = np.where(m.astype(bool), np.exp(s - lse[0, 0][:, None]), 0.0)
    assert np.abs(P.sum(1) - 1).max() < 1e-13
    assert np.abs(P @ v[0, 0].astype(np.float64) - out[0, 0]).max() < 1e-13
    # adding one vector c to every key shifts each row's scores by a constant: out unchanged
    c = np.linspace(-1, 1, D).astype(np.float32)
    out2, lse2 = O.fwd(q, k + c, v, p["sink"], p["window"])
    assert np.abs(out2 - out).max() < 1e-6       # k + c is rounded to float32
    # dead keys never matter: poison them for the last row and look at that row only
    k3, v3 = k.copy(), v.copy()
    dead = np.where(m[N - 1] == 0)[0]
    k3[0, 0, dead] = np.nan
    v3[0, 0, dead] = np.inf
    out3, lse3 = O.fwd(q, k3, v3, p["sink"], p["window"], rows=(N - 1, N))
    assert np.array_equal(out3[0, 0, N - 1], out[0, 0, N - 1]) and lse3[0, 0, N - 1] == lse[0, 0, N - 1]


def autograd_reference(q, k, v, dout, mask):
    tq, tk, tv = (torch.tensor(np.asarray(x, np.float64), requires_grad=True) for x in (q, k, v))
    G = tq.shape[1] // tk.shape[1]
    o = F.scaled_dot_product_attention(tq, tk.repeat_interleave(G, 1), tv.repeat_interleave(G, 1),
                                       attn_mask=torch.as_tensor(mask.astype(bool)))
    o.backward(torch.as_tensor(np.asarray(dout, np.float64)))
    return tq.grad.numpy(), tk.grad.numpy(), tv.grad.numpy()


@pytest.mark.parametrize("name", GOLDEN_MASKS)
def test_bwd_matches_library_autograd_on_hand_written_masks(name):
    p, m = load_golden_mask(name)
    q, k, v, g = inputs(2, 4, 2, p["N"], 8, seed=21, with_dout=True)
    r = O.bwd(q, k, v, g, p["sink"], p["window"], p["block"], p["stride"])
    dq, dk, dv = autograd_reference(q, k, v, g, m)
    assert np.abs(r["dq"] - dq).max() < 1e-12
    assert np.abs(r["dk"] - dk).max() < 1e-12
    assert np.abs(r["dv"] - dv).max() < 1e-12


def test_bwd_medium_gqa_matches_autograd():
    N, D = 96, 16
    q, k, v, g = inputs(1, 4, 2, N, D, seed=22, with_dout=True)
    r = O.bwd(q, k, v, g, 4, 20)
    dq, dk, dv = autograd_reference(q, k, v, g, token_mask(N, 4, 20))
    for a, b in ((r["dq"], dq), (r["dk"], dk), (r["dv"], dv)):
        assert np.abs(a - b).max() < 1e-12


def test_bwd_finite_differences():
    p, _ = load_golden_mask("mask_block_strided.txt")
    N, D = p["N"], 4
    q, k, v, g = inputs(1, 2, 1, N, D, seed=23, with_dout=True)
    args = (p["sink"], p["window"], p["block"], p["stride"])
    r = O.bwd(q, k, v, g, *args)

    def loss(q_, k_, v_):
        o, _ = O.fwd(q_, k_, v_, *args)
        return float((o * g.astype(np.float64)).sum())

    eps = 2.0 ** -7     # exactly representable steps keep the float32 inputs exact
    rng = np.random.default_rng(1)
    for name, arr, grad in (("q", q, r["dq"]), ("k", k, r["dk"]), ("v", v, r["dv"])):
        for _ in range(12):
            idx = tuple(rng.integers(0, s) for s in arr.shape)
            hi, lo = arr.copy(), arr.copy()
            hi[idx] += eps
            lo[idx] -= eps
            a = dict(q=q, k=k, v=v)
            a[name] = hi
            fp = loss(a["q"], a["k"], a["v"])
            a[name] = lo
            fm = loss(a["q"], a["k"], a["v"])
            fd = (fp - fm) / (hi[idx].astype(np.float64) - lo[idx].astype(np.float64))
            assert abs(fd - grad[idx]) < 2e-4 * max(1.0, abs(grad[idx])), (name, idx, fd, grad[idx])


def test_bwd_invariants():
    p, m = load_golden_mask("mask_sink_window_token.txt")
    N, D = p["N"], 8
    q, k, v, g = inputs(1, 2, 2, N, D, seed=24, with_dout=True)
    r = O.bwd(q, k, v, g, p["sink"], p["window"])
    # each row's dS sums to zero, hence the key gradients of a head sum to zero
    assert np.abs(r["dk"].sum(axis=2)).max() < 1e-13
    # dv sums to the P-weighted column mass: sum_j dv_j = sum_i dout_i
    assert np.abs(r["dv"].sum(axis=2) - g.astype(np.float64).sum(axis=2)).max() < 1e-13
    # zero upstream gradient on all but a few rows: keys dead for those rows get exactly zero
    rows = [6, 9]
    g2 = np.zeros_like(g)
    g2[:, :, rows] = g[:, :, rows]
    r2 = O.bwd(q, k, v, g2, p["sink"], p["window"])
    touched = m[rows].any(axis=0)
    assert np.all(r2["dk"][:, :, ~touched] == 0) and np.all(r2["dv"][:, :, ~touched] == 0)
    assert np.all(np.abs(r2["dv"][:, :, touched]).sum(-1) > 0)
    other = [i for i in range(N) if i not in rows]
    assert np.all(r2["dq"][:, :, other] == 0)
    assert np.all(O.bwd(q, k, v, np.zeros_like(g), p["sink"], p["window"])["dq"] == 0)


def test_gqa_equals_explicit_repetition():
    N, D = 40, 8
    q, k, v, g = inputs(1, 6, 2, N, D, seed=25, with_dout=True)
    a = O.bwd(q, k, v, g, 3, 9)
    krep, vrep = np.repeat(k, 3, axis=1), np.repeat(v, 3, axis=1)
    b = O.bwd(q, krep, vrep, g, 3, 9)
    assert np.abs(a["out"] - b["out"]).max() < 1e-14
    assert np.abs(a["dq"] - b["dq"]).max() < 1e-14
    assert np.abs(a["dk"] - b["dk"].reshape(1, 2, 3, N, D).sum(2)).max() < 1e-13
    assert np.abs(a["dv"] - b["dv"].reshape(1, 2, 3, N, D).sum(2)).max() < 1e-13


@pytest.mark.parametrize("N", [1, 3, 5, 6, 17, 40])
def test_decode_equals_last_prefill_row_and_library_attention(N):
    sink, window, D = 2, 3, 8
    q, k, v = inputs(2, 4, 2, N, D, seed=30 + N)
    kc, vc = O.build_ring_cache(k, v, sink, window)
    qlast = q[:, :, N - 1]
    out, lse = O.decode(qlast, kc, vc, N, sink, window)
    fo, fl = O.fwd(q, k, v, sink, window, rows=(N - 1, N))
    assert np.abs(out - fo[:, :, N - 1]).max() < 1e-13
    assert np.abs(lse - fl[:, :, N - 1]).max() < 1e-13
    # library attention over the gathered live keys
    livej = [j for j in range(N) if j < sink or N - 1 - j < window]
    want = sdpa(qlast[:, :, None], k[:, :, livej], v[:, :, livej]).numpy()[:, :, 0]
    assert np.abs(out - want).max() < 1e-13


def test_decode_invariant_under_slot_permutation():
    sink, window, D, N = 4, 12, 16, 100
    q, kc, vc = (x.numpy() for x in lg_synth.decode_inputs(2, 4, 4, sink + window, D, seed=41))
    out, lse = O.decode(q, kc, vc, N, sink, window)
    perm = np.random.default_rng(2).permutation(sink + window)
    out2, lse2 = O.decode(q, kc[:, :, perm], vc[:, :, perm], N, sink, window)
    assert np.abs(out - out2).max() < 1e-13 and np.abs(lse - lse2).max() < 1e-13
    # partial fill: only the first N slots count
    kc3, vc3 = kc.copy(), vc.copy()
    kc3[:, :, 5:] = np.nan
    vc3[:, :, 5:] = np.nan
    out3, _ = O.decode(q, kc3, vc3, 5, sink, window)
    want = sdpa(q[:, :, None], kc[:, :, :5], vc[:, :, :5]).numpy()[:, :, 0]
    assert np.abs(out3 - want).max() < 1e-13


def test_partial_backward_equals_slices_of_the_full_one():
    N, D = 120, 8
    q, k, v, g = inputs(1, 4, 2, N, D, seed=26, with_dout=True)
    full = O.bwd(q, k, v, g, 6, 20, 2, 9)
    part = O.bwd(q, k, v, g, 6, 20, 2, 9, rows=(50, 71), keys=(3, 30))
    assert np.array_equal(part["dq"][:, :, 50:71], full["dq"][:, :, 50:71])
    assert np.array_equal(part["dk"][:, :, 3:30], full["dk"][:, :, 3:30])
    assert np.array_equal(part["dv"][:, :, 3:30], full["dv"][:, :, 3:30])
    assert np.isnan(part["dq"][:, :, :50]).all() and np.isnan(part["dk"][:, :, 30:]).all()
