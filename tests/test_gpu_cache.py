"""GPU parity of the reduced-KV-cache calls through the C ABI:
lg_kv_ring_append (bit-exact against the oracle's append) and lg_sparse_attn_decode_cache
(against row N-1 of the oracle's forward on the whole context) for sink+window, block-granular
and block-strided patterns."""
import numpy as np
import pytest
import torch

import lg_synth
import paper_2410_01485_amd as lg
from gpu_util import DEV, TOL_LSE, TOL_OUT, TOL_REL, assert_close, f32np
from oracle import lg_oracle as O

pytestmark = pytest.mark.gpu

PATTERNS = [
    # N, sink, window, block, stride
    (1, 4, 8, 1, 0), (13, 4, 8, 1, 0), (300, 16, 128, 1, 0),
    (65, 16, 32, 16, 0), (207, 16, 48, 16, 0), (207, 16, 48, 16, 4), (256, 16, 16, 16, 2), (257, 16, 16, 16, 2),
    (1000, 64, 192, 64, 8), (1000, 64, 128, 64, 3), (97, 4, 8, 1, 5), (300, 8, 24, 8, 1), (3000, 64, 256, 64, 4),
]


def bits(t):
    """Raw bytes of a tensor as a numpy integer array (bf16 has no numpy dtype)."""
    return t.detach().cpu().contiguous().view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32).numpy()


def chunking(N, seed):
    rng = np.random.default_rng(seed)
    out, left = [], N
    while left > 0:
        T = int(min(left, rng.integers(1, max(2, N // 2))))
        out.append(T)
        left -= T
    return out


def gpu_append_all(k, v, sink, window, block, stride, chunks, slots, fill):
    B, H, N, D = k.shape
    kc = torch.full((B, H, slots, D), fill, dtype=k.dtype, device=DEV)
    vc = torch.full((B, H, slots, D), -fill, dtype=k.dtype, device=DEV)
    kd, vd = k.to(DEV), v.to(DEV)
    pos = 0
    for T in chunks:
        lg.lg_kv_ring_append(kd[:, :, pos:pos + T].contiguous(), vd[:, :, pos:pos + T].contiguous(), kc, vc, pos,
                             sink, window, block, stride)
        pos += T
    torch.cuda.synchronize()
    return kc, vc


def oracle_append_all(k, v, sink, window, block, stride, slots, fill):
    kb, vb = bits(k), bits(v)
    B, H, N, D = kb.shape
    fk = bits(torch.full((1,), fill, dtype=k.dtype))[0]
    fv = bits(torch.full((1,), -fill, dtype=k.dtype))[0]
    kc = np.full((B, H, slots, D), fk, dtype=kb.dtype)
    vc = np.full((B, H, slots, D), fv, dtype=vb.dtype)
    O.ring_append(kb, kc, 0, sink, window, block, stride)
    O.ring_append(vb, vc, 0, sink, window, block, stride)
    return kc, vc


@pytest.mark.parametrize("dtype,D", [(torch.bfloat16, 128), (torch.bfloat16, 64), (torch.float32, 128), (torch.float32, 64)])
@pytest.mark.parametrize("N,sink,window,block,stride", PATTERNS)
def test_append_is_bit_exact(dtype, D, N, sink, window, block, stride):
    _, k, v = lg_synth.prefill_inputs(2, 3, 3, N, D, 31 + N, dtype)
    slots = lg.lg_kv_cache_slots(N, sink, window, block, stride) + 5  # spare slots must stay untouched
    for chunks in ([N], chunking(N, N), [1] * N if N <= 100 else chunking(N, 2 * N)):
        kc, vc = gpu_append_all(k, v, sink, window, block, stride, chunks, slots, 7.0)
        wk, wv = oracle_append_all(k, v, sink, window, block, stride, slots, 7.0)
        assert np.array_equal(bits(kc), wk), ("k cache", chunks[:4])
        assert np.array_equal(bits(vc), wv), ("v cache", chunks[:4])


def decode_cache(q, kc, vc, N, sink, window, block, stride):
    B, Hq, D = q.shape
    Hkv = kc.shape[1]
    code = lg.LG_BF16 if q.dtype == torch.bfloat16 else lg.LG_F32
    need = lg.decode_cache_workspace_bytes(B, Hq, Hkv, N, D, sink, window, block, stride, code)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=DEV)
    out = torch.full_like(q, float("nan"))
    lse = torch.full((B, Hq), float("nan"), dtype=torch.float32, device=DEV)
    lg.lg_sparse_attn_decode_cache(q, kc, vc, out, lse, ws, N, sink, window, block, stride)
    torch.cuda.synchronize()
    return out, lse


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("N,sink,window,block,stride", PATTERNS)
def test_decode_over_cache_equals_last_prefill_row(dtype, N, sink, window, block, stride):
    B, Hq, Hkv, D = 2, 4, 2, 128
    q, k, v = lg_synth.prefill_inputs(B, Hq, Hkv, N, D, 57 + N, dtype)
    slots = lg.lg_kv_cache_slots(N, sink, window, block, stride)
    # unwritten and dead slots hold large values that would wreck the result if they were read
    kc, vc = gpu_append_all(k, v, sink, window, block, stride, chunking(N, N + 1), slots, 1.0e4)
    out, lse = decode_cache(q[:, :, N - 1].contiguous().to(DEV), kc, vc, N, sink, window, block, stride)
    wo, wl = O.fwd(f32np(q), f32np(k), f32np(v), sink, window, block, stride, rows=(N - 1, N))
    tag = "decode_cache N%d s%d w%d b%d st%d %s" % (N, sink, window, block, stride, dtype)
    assert_close(f32np(out), wo[:, :, N - 1], TOL_OUT[dtype], TOL_REL[dtype], tag + " out")
    assert_close(f32np(lse), wl[:, :, N - 1], TOL_LSE[dtype], None, tag + " lse")


def test_generation_loop_block_strided():
    # prefill 500 tokens, then 140 single-token steps (crossing block and stride boundaries):
    # every step appends one token and must reproduce that row of the forward on the whole context
    B, Hq, Hkv, D, sink, window, block, stride = 1, 4, 4, 64, 32, 64, 32, 3
    N0, steps = 500, 140
    q, k, v = lg_synth.prefill_inputs(B, Hq, Hkv, N0 + steps, D, 77, torch.bfloat16)
    wo, wl = O.fwd(f32np(q), f32np(k), f32np(v), sink, window, block, stride, rows=(N0, N0 + steps))
    slots = lg.lg_kv_cache_slots(N0 + steps, sink, window, block, stride)
    kd, vd, qd = k.to(DEV), v.to(DEV), q.to(DEV)
    kc = torch.full((B, Hkv, slots, D), 1.0e4, dtype=torch.bfloat16, device=DEV)
    vc = torch.full_like(kc, -1.0e4)
    lg.lg_kv_ring_append(kd[:, :, :N0].contiguous(), vd[:, :, :N0].contiguous(), kc, vc, 0, sink, window, block, stride)
    for t in range(N0, N0 + steps):
        lg.lg_kv_ring_append(kd[:, :, t:t + 1].contiguous(), vd[:, :, t:t + 1].contiguous(), kc, vc, t, sink, window,
                             block, stride)
        out, lse = decode_cache(qd[:, :, t].contiguous(), kc, vc, t + 1, sink, window, block, stride)
        assert_close(f32np(out), wo[:, :, t], TOL_OUT[torch.bfloat16], TOL_REL[torch.bfloat16], "step %d out" % t)
        assert_close(f32np(lse), wl[:, :, t], TOL_LSE[torch.bfloat16], None, "step %d lse" % t)


@pytest.mark.parametrize("sink,window,block,stride", [(64, 2048, 64, 0), (64, 2048, 64, 64), (0, 64, 64, 64)])
def test_paper_settings_full_context(sink, window, block, stride):
    # Section 4.1 settings at 128K: attention sink (1 sink block + 32 local blocks), block sparse
    # (one retained block per 64), and the two combined; two heads, cache built in one append
    B, H, D, N = 1, 2, 128, 131072
    q, k, v = lg_synth.prefill_inputs(B, H, H, N, D, 91, torch.bfloat16)
    slots = lg.lg_kv_cache_slots(N, sink, window, block, stride)
    kc, vc = gpu_append_all(k, v, sink, window, block, stride, [N], slots, 1.0e4)
    wk, wv = oracle_append_all(k, v, sink, window, block, stride, slots, 1.0e4)
    assert np.array_equal(bits(kc), wk) and np.array_equal(bits(vc), wv)
    out, lse = decode_cache(q[:, :, N - 1].contiguous().to(DEV), kc, vc, N, sink, window, block, stride)
    wo, wl = O.fwd(f32np(q), f32np(k), f32np(v), sink, window, block, stride, rows=(N - 1, N))
    assert_close(f32np(out), wo[:, :, N - 1], TOL_OUT[torch.bfloat16], TOL_REL[torch.bfloat16], "paper setting out")
    assert_close(f32np(lse), wl[:, :, N - 1], TOL_LSE[torch.bfloat16], None, "paper setting lse")


# ------------------------------------------------------------------ paged cache, per-sequence lengths
def paged_setup(lens, Hq, Hkv, D, sink, window, block, stride, page_size, dtype, seed):
    """Contexts of different lengths, a page table that scatters every sequence's pages over the pool."""
    B, n_max = len(lens), max(lens) + 8
    slots = lg.lg_kv_cache_slots(n_max, sink, window, block, stride)
    pps = (slots + page_size - 1) // page_size
    num_pages = B * pps + 3
    perm = np.random.default_rng(seed).permutation(num_pages)[:B * pps].reshape(B, pps).astype(np.int32)
    table = torch.as_tensor(perm).to(DEV)
    kp = torch.full((num_pages, Hkv, page_size, D), 1.0e4, dtype=dtype, device=DEV)
    vp = torch.full_like(kp, -1.0e4)
    ctx = [lg_synth.prefill_inputs(1, Hq, Hkv, n, D, seed + 13 * b, dtype) for b, n in enumerate(lens)]
    return n_max, table, kp, vp, ctx


def paged_decode(qs, kp, vp, table, lens, n_max, sink, window, block, stride):
    q = torch.stack(qs).to(DEV)
    B, Hq, D = q.shape
    Hkv = kp.shape[1]
    code = lg.LG_BF16 if q.dtype == torch.bfloat16 else lg.LG_F32
    need = lg.decode_paged_workspace_bytes(B, Hq, Hkv, n_max, D, sink, window, block, stride, code)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=DEV)
    out = torch.full_like(q, float("nan"))
    lse = torch.full((B, Hq), float("nan"), dtype=torch.float32, device=DEV)
    sl = torch.as_tensor(np.asarray(lens, dtype=np.int32)).to(DEV)
    lg.lg_sparse_attn_decode_paged(q, kp, vp, table, sl, out, lse, ws, n_max, sink, window, block, stride)
    torch.cuda.synchronize()
    return out, lse


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("sink,window,block,stride,page_size", [
    (16, 128, 1, 0, 16), (64, 192, 64, 8, 64), (16, 48, 16, 4, 32), (0, 64, 64, 2, 256)])
def test_paged_varlen_decode(dtype, sink, window, block, stride, page_size):
    lens = [1000, 37, 700, 1, 333]
    Hq, Hkv, D = 4, 2, 128
    n_max, table, kp, vp, ctx = paged_setup(lens, Hq, Hkv, D, sink, window, block, stride, page_size, dtype, 5)
    for b, (q, k, v) in enumerate(ctx):  # fill sequence b's pages in a few append calls
        pos = 0
        for T in chunking(lens[b], 100 + b):
            lg.lg_kv_paged_append(k[:, :, pos:pos + T].contiguous().to(DEV), v[:, :, pos:pos + T].contiguous().to(DEV),
                                  kp, vp, table[b:b + 1], torch.tensor([pos], dtype=torch.int32, device=DEV), n_max,
                                  sink, window, block, stride)
            pos += T
    # the pages of a sequence, gathered through its table row, are the oracle's cache row
    slots = lg.lg_kv_cache_slots(n_max, sink, window, block, stride)
    for b, (q, k, v) in enumerate(ctx):
        wk, wv = oracle_append_all(k, v, sink, window, block, stride, slots, 1.0e4)
        got = bits(kp[table[b].long()].permute(1, 0, 2, 3).reshape(Hkv, -1, D)[:, :slots])
        assert np.array_equal(got, wk[0]), "pages of sequence %d" % b
    out, lse = paged_decode([q[0, :, n - 1] for (q, _, _), n in zip(ctx, lens)], kp, vp, table, lens, n_max, sink,
                            window, block, stride)
    for b, ((q, k, v), n) in enumerate(zip(ctx, lens)):
        wo, wl = O.fwd(f32np(q), f32np(k), f32np(v), sink, window, block, stride, rows=(n - 1, n))
        assert_close(f32np(out[b]), wo[0, :, n - 1], TOL_OUT[dtype], TOL_REL[dtype], "paged seq %d out" % b)
        assert_close(f32np(lse[b]), wl[0, :, n - 1], TOL_LSE[dtype], None, "paged seq %d lse" % b)


def test_paged_generation_step_all_sequences_at_once():
    # every sequence appends one token at its own position in ONE call, then decodes at its own length
    sink, window, block, stride, page_size = 32, 64, 32, 3, 64
    lens = [400, 95, 250]
    Hq, Hkv, D, steps = 4, 4, 64, 70
    dtype = torch.bfloat16
    full = [n + steps for n in lens]
    n_max, table, kp, vp, ctx = paged_setup(full, Hq, Hkv, D, sink, window, block, stride, page_size, dtype, 9)
    for b, (q, k, v) in enumerate(ctx):
        lg.lg_kv_paged_append(k[:, :, :lens[b]].contiguous().to(DEV), v[:, :, :lens[b]].contiguous().to(DEV), kp, vp,
                              table[b:b + 1], torch.zeros(1, dtype=torch.int32, device=DEV), n_max, sink, window,
                              block, stride)
    want = [O.fwd(f32np(q), f32np(k), f32np(v), sink, window, block, stride, rows=(lens[b], lens[b] + steps))
            for b, (q, k, v) in enumerate(ctx)]
    for s in range(steps):
        pos = [n + s for n in lens]
        kn = torch.stack([k[0, :, p:p + 1] for (_, k, _), p in zip(ctx, pos)]).to(DEV)
        vn = torch.stack([v[0, :, p:p + 1] for (_, _, v), p in zip(ctx, pos)]).to(DEV)
        lg.lg_kv_paged_append(kn, vn, kp, vp, table, torch.as_tensor(np.asarray(pos, dtype=np.int32)).to(DEV), n_max,
                              sink, window, block, stride)
        out, lse = paged_decode([q[0, :, p] for (q, _, _), p in zip(ctx, pos)], kp, vp, table, [p + 1 for p in pos],
                                n_max, sink, window, block, stride)
        for b, p in enumerate(pos):
            assert_close(f32np(out[b]), want[b][0][0, :, p], TOL_OUT[dtype], TOL_REL[dtype], "step %d seq %d out" % (s, b))
            assert_close(f32np(lse[b]), want[b][1][0, :, p], TOL_LSE[dtype], None, "step %d seq %d lse" % (s, b))
