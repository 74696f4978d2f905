"""GPU parity of the packed, different-lengths prefill calls (lg_sparse_attn_fwd_varlen /
lg_sparse_attn_bwd_varlen, through the C ABI): every sequence of the pack against the fp64 oracle run on
that sequence alone (the plain definition: sequences do not see each other), and against the fixed-length
entry points on a copy of the sequence (same kernels at the same length: identical bits wherever those are
reproducible)."""
import numpy as np
import pytest
import torch

import lg_synth
import paper_2410_01485_amd as lg
from gpu_util import DEV, TOL_LSE, TOL_OUT, TOL_REL, assert_close, dq_delta_allowance, f32np
from oracle import lg_oracle as O

pytestmark = pytest.mark.gpu


def pack(lens, Hq, Hkv, D, dtype, seed):
    """Seeded sequences, each drawn on its own, laid side by side per head: q, g [Hq,T,D], k, v [Hkv,T,D];
    also returns the per-sequence tensors ([1,H,n,D]) and the offsets."""
    seqs = [lg_synth.prefill_inputs(1, Hq, Hkv, max(n, 1), D, seed + 17 * s, dtype, with_dout=True)
            for s, n in enumerate(lens)]
    seqs = [tuple(t[:, :, :n] for t in tup) for tup, n in zip(seqs, lens)]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(int).tolist()
    packed = [torch.cat([tup[x][0] for tup in seqs], dim=1).contiguous() for x in range(4)]
    return packed, seqs, cu


def run_varlen(packed, cu, sink, window, block, stride, scale=0.0):
    q, k, v, g = (t.to(DEV) for t in packed)
    Hq, T, D = q.shape
    Hkv = k.shape[0]
    code = lg.LG_BF16 if q.dtype == torch.bfloat16 else lg.LG_F32
    out = torch.full_like(q, float("nan"))
    lse = torch.full((Hq, T), float("nan"), dtype=torch.float32, device=DEV)
    lg.lg_sparse_attn_fwd_varlen(q, k, v, out, lse, cu, sink, window, block, stride, scale)
    need = lg.bwd_varlen_workspace_bytes(cu, Hq, Hkv, D, sink, window, block, stride, code)
    lens = np.diff(cu)
    assert need == max([256] + [lg.bwd_workspace_bytes(1, Hq, Hkv, int(n), D, sink, window, block, stride, code)
                                for n in lens if n > 0])
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    dq, dk, dv = (torch.full_like(t, float("nan")) for t in (q, k, v))
    lg.lg_sparse_attn_bwd_varlen(q, k, v, out, lse, g, dq, dk, dv, ws, cu, sink, window, block, stride, scale)
    torch.cuda.synchronize()
    return out, lse, dq, dk, dv


def run_fixed(seq, sink, window, block, stride, scale=0.0):
    """The fixed-length entry points on one sequence [1,H,n,D]."""
    q, k, v, g = (t.contiguous().to(DEV) for t in seq)
    _, Hq, n, D = q.shape
    Hkv = k.shape[1]
    code = lg.LG_BF16 if q.dtype == torch.bfloat16 else lg.LG_F32
    out = torch.empty_like(q)
    lse = torch.empty(1, Hq, n, dtype=torch.float32, device=DEV)
    lg.lg_sparse_attn_fwd(q, k, v, out, lse, sink, window, block, stride, scale)
    ws = torch.empty(lg.bwd_workspace_bytes(1, Hq, Hkv, n, D, sink, window, block, stride, code), dtype=torch.uint8,
                     device=DEV)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    lg.lg_sparse_attn_bwd(q, k, v, out, lse, g, dq, dk, dv, ws, sink, window, block, stride, scale)
    torch.cuda.synchronize()
    return out[0], lse[0], dq[0], dk[0], dv[0]


def check_pack(lens, Hq, Hkv, D, sink, window, block, stride, dtype, seed, oracle_rows=None):
    packed, seqs, cu = pack(lens, Hq, Hkv, D, dtype, seed)
    got = run_varlen(packed, cu, sink, window, block, stride)
    atomics = stride > 0 or Hq != Hkv    # dk / dv of column keys are summed with float atomics then
    names = ("out", "lse", "dq", "dk", "dv")
    for s, n in enumerate(lens):
        if n == 0:
            continue
        a, b = cu[s], cu[s + 1]
        mine = [t[:, a:b] for t in got]
        tag = "varlen seq %d (n=%d) of %s Hq%d Hkv%d D%d s%d w%d b%d st%d %s" % (
            s, n, list(lens), Hq, Hkv, D, sink, window, block, stride, dtype)
        fixed = run_fixed(seqs[s], sink, window, block, stride)
        for name, x, y in zip(names, mine, fixed):
            if name in ("dk", "dv") and atomics and dtype == torch.bfloat16:
                assert torch.allclose(x.float(), y.float(), rtol=2e-2, atol=2e-2), tag + " " + name
            else:
                assert torch.equal(x, y), tag + " " + name + " differs from the fixed-length call"
        q, k, v, g = (f32np(t) for t in seqs[s])
        if oracle_rows is not None and n > oracle_rows:   # long sequences: the forward on sampled rows
            rows = np.unique(np.concatenate([np.arange(0, 40), np.arange(n - 40, n),
                                             np.random.default_rng(seed + s).integers(0, n, 200)]))
            for r0 in rows[::16]:
                wo, wl = O.fwd(q, k, v, sink, window, block, stride, rows=(int(r0), int(r0) + 1))
                assert_close(f32np(mine[0])[None][:, :, r0], wo[:, :, r0], TOL_OUT[dtype], TOL_REL[dtype], tag + " out")
                assert_close(f32np(mine[1])[None][:, :, r0], wl[:, :, r0], TOL_LSE[dtype], None, tag + " lse")
            continue
        w = O.bwd(q, k, v, g, sink, window, block, stride)
        allow = None
        if dtype == torch.bfloat16:
            allow = dq_delta_allowance(q, k, g, w["out"], sink, window, block, stride)
        assert_close(f32np(mine[0])[None], w["out"], TOL_OUT[dtype], TOL_REL[dtype], tag + " out")
        assert_close(f32np(mine[1])[None], w["lse"], TOL_LSE[dtype], None, tag + " lse")
        for name, x in zip(names[2:], mine[2:]):
            # where every row has a single live key (a one-token sequence, the diagonal-only pattern) dq and
            # dk are zero by cancellation (dP = Delta exactly): what is left is the rounding of two dot
            # products summed in different orders, judged by the absolute bound alone
            rel = None if np.abs(w[name]).max() < 1e-12 else TOL_REL[dtype]
            assert_close(f32np(x)[None], w[name], TOL_OUT[dtype], rel, tag + " " + name,
                         allow=allow if name == "dq" else None)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("D", [64, 128])
def test_ragged_pack_sink_window_gqa(dtype, D):
    # lengths below, at and above the tiles' sizes, a single token, an empty sequence in the middle
    check_pack([300, 1, 0, 777, 64, 1500, 257], 4, 2, D, 16, 200, 1, 0, dtype, 401)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("lens,sink,window,block,stride", [
    ([1024, 130, 900], 64, 192, 64, 8),      # block-granular with strided columns (column parts, atomics)
    ([1000, 47, 480], 48, 96, 48, 3),        # a block that is not a power of two
    ([5, 0, 0, 9], 0, 1, 1, 0),              # the diagonal only; empty sequences at both kinds of places
    ([640, 333], 5, 100000, 1, 0),           # window beyond every length: plain causal attention
])
def test_ragged_pack_patterns(dtype, lens, sink, window, block, stride):
    check_pack(lens, 2, 1, 128, sink, window, block, stride, dtype, 402)


@pytest.mark.parametrize("D,sink,window,block,stride", [(128, 16, 100, 1, 0), (64, 64, 128, 64, 2)])
def test_many_short_sequences_in_shared_launches(D, sink, window, block, stride):
    """300 requests of 0 .. 400 tokens: the bf16 forward puts up to 128 sequences into one launch (every
    (sequence, head, query tile) a workgroup of the same grid) and derives each sequence's pattern on the device.
    Every sequence against the oracle on it alone; a sample of them bit for bit against the fixed-length call."""
    rng = np.random.default_rng(405)
    lens = [int(x) for x in rng.integers(0, 401, 300)]
    lens[7] = lens[130] = lens[299] = 0
    lens[128] = 1
    Hq, Hkv, dt = 4, 2, torch.bfloat16
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(int).tolist()
    T = cu[-1]
    q, k, v = (t[0] for t in lg_synth.prefill_inputs(1, Hq, Hkv, T, D, 406, dt, device=DEV))
    out = torch.full_like(q, float("nan"))
    lse = torch.full((Hq, T), float("nan"), dtype=torch.float32, device=DEV)
    lg.lg_sparse_attn_fwd_varlen(q, k, v, out, lse, cu, sink, window, block, stride)
    torch.cuda.synchronize()
    assert not torch.isnan(out.float()).any() and not torch.isnan(lse).any()
    qn, kn, vn, on, ln = (f32np(t) for t in (q, k, v, out, lse))
    for s, n in enumerate(lens):
        if n == 0:
            continue
        a, b = cu[s], cu[s + 1]
        wo, wl = O.fwd(qn[None, :, a:b], kn[None, :, a:b], vn[None, :, a:b], sink, window, block, stride)
        tag = "short sequence %d (n=%d) D%d s%d w%d b%d st%d" % (s, n, D, sink, window, block, stride)
        assert_close(on[None, :, a:b], wo, TOL_OUT[dt], TOL_REL[dt], tag + " out")
        assert_close(ln[None, :, a:b], wl, TOL_LSE[dt], None, tag + " lse")
        if s % 37 == 0 or s in (127, 128, 129, 298):
            o1 = torch.empty(1, Hq, n, D, dtype=dt, device=DEV)
            l1 = torch.empty(1, Hq, n, dtype=torch.float32, device=DEV)
            lg.lg_sparse_attn_fwd(q[None, :, a:b].contiguous(), k[None, :, a:b].contiguous(),
                                  v[None, :, a:b].contiguous(), o1, l1, sink, window, block, stride)
            torch.cuda.synchronize()
            assert torch.equal(o1[0], out[:, a:b]) and torch.equal(l1[0], lse[:, a:b]), tag


def test_long_sequences_take_the_resident_kernels():
    """Head dim 128, window 4096: the sequences of 5000 and 9000 tokens run the 64-rows-per-wave backward
    kernels (one resident workgroup per CU, work queue in the shared workspace, cleared per sequence), the
    700-token one in between the same instances at a short length.  No GQA, no stride: everything is
    bit-reproducible, so the whole pack must equal the fixed-length calls bit for bit; forward rows of the
    long sequences are sampled against the oracle, the short one is compared in full."""
    check_pack([5000, 700, 9000], 2, 2, 128, 64, 4096, 1, 0, torch.bfloat16, 403, oracle_rows=2000)


def test_neighbours_in_the_pack_do_not_matter():
    """A sequence's results do not depend on what is packed around it: the neighbours are replaced by values
    that would wreck them if read (Inf in V, huge K, Q and dO), the middle sequence comes out bit-identical.
    Every output row belongs to some sequence, so nothing of the NaN fill survives a call."""
    dt, Hq, Hkv, D, sink, window = torch.bfloat16, 2, 2, 128, 16, 300
    lens = [500, 321, 700]
    packed, seqs, cu = pack(lens, Hq, Hkv, D, dt, 404)
    ref = run_varlen(packed, cu, sink, window, 1, 0)
    for t in ref:
        assert not torch.isnan(t.float()).any()
    q, k, v, g = (t.clone() for t in packed)
    a, b = cu[1], cu[2]
    for t, val in ((q, 50.0), (k, 300.0), (v, float("inf")), (g, -70.0)):
        t[:, :a] = val
        t[:, b:] = val
    got = run_varlen([q, k, v, g], cu, sink, window, 1, 0)
    for x, y, name in zip(got, ref, ("out", "lse", "dq", "dk", "dv")):
        assert torch.equal(x[:, a:b], y[:, a:b]), name


def test_serving_mix_full_size_sampled():
    """The pack the benchmark times: eight requests of 2K .. 64K tokens, 32 heads, D=128, sink 64 + window 4096,
    forward and backward.  The oracle recomputes sampled query rows (out, lse, dq) and sampled keys (dk, dv) of
    single heads on the sequence alone: the start of the longest request with its sink keys (seen by 65536 rows),
    where a request's window starts to slide, steady state in a request in the middle of the pack, a request
    shorter than the window, and the last rows of the pack."""
    lens = [2048, 4096, 8192, 12288, 16384, 24576, 32768, 65536]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(int).tolist()
    H, D, sink, window, T = 32, 128, 64, 4096, cu[-1]
    q, k, v, g = (t[0] for t in lg_synth.prefill_inputs(1, H, H, T, D, 20241012, torch.bfloat16, with_dout=True,
                                                        device=DEV))
    out = torch.empty_like(q)
    lse = torch.empty(H, T, dtype=torch.float32, device=DEV)
    lg.lg_sparse_attn_fwd_varlen(q, k, v, out, lse, cu, sink, window)
    ws = torch.empty(lg.bwd_varlen_workspace_bytes(cu, H, H, D, sink, window, 1, 0, lg.LG_BF16), dtype=torch.uint8,
                     device=DEV)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    lg.lg_sparse_attn_bwd_varlen(q, k, v, out, lse, g, dq, dk, dv, ws, cu, sink, window)
    torch.cuda.synchronize()
    for t in (out, dq, dk, dv):
        assert torch.isfinite(t.float()).all()
    tol, rel = TOL_OUT[torch.bfloat16], TOL_REL[torch.bfloat16]
    for h, s, rows, keys in ((0, 7, (0, 40), (0, 40)),                       # longest request: first rows, sink keys
                             (5, 7, (4080, 4120), (4140, 4180)),             # its window starts to slide
                             (13, 5, (20001, 20041), (15000, 15040)),        # steady state, a request inside the pack
                             (21, 0, (2008, 2048), (1000, 1040)),            # a request shorter than the window
                             (31, 7, (65496, 65536), (65496, 65536))):       # the last rows of the pack
        print("head", h, "sequence", s, "rows", rows, "keys", keys, flush=True)
        a0, a1 = cu[s], cu[s + 1]
        a = [f32np(x[h:h + 1, a0:a1])[None] for x in (q, k, v, g)]
        w = O.bwd(*a, sink, window, rows=rows, keys=keys)
        al = dq_delta_allowance(a[0], a[1], a[3], w["out"], sink, window, rows=rows)
        tag = "serving mix h%d seq%d " % (h, s)
        r0, r1, k0, k1 = rows[0], rows[1], keys[0], keys[1]
        assert_close(f32np(dq[h, a0 + r0:a0 + r1]), w["dq"][0, 0, r0:r1], tol, rel, tag + "dq", allow=al[0, 0, r0:r1])
        assert_close(f32np(dk[h, a0 + k0:a0 + k1]), w["dk"][0, 0, k0:k1], tol, rel, tag + "dk")
        assert_close(f32np(dv[h, a0 + k0:a0 + k1]), w["dv"][0, 0, k0:k1], tol, rel, tag + "dv")
        assert_close(f32np(out[h, a0 + r0:a0 + r1]), w["out"][0, 0, r0:r1], tol, rel, tag + "out")
        assert_close(f32np(lse[h, a0 + r0:a0 + r1]), w["lse"][0, 0, r0:r1], TOL_LSE[torch.bfloat16], None, tag + "lse")
