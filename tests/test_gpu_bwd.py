"""GPU parity: lg_sparse_attn_bwd (through the C ABI) against the fp64 oracle, element by element.

The GPU backward consumes the GPU forward's own out / lse (as a training step does); the oracle
computes its forward in fp64 itself."""
import numpy as np
import pytest
import torch

import lg_synth
import paper_2410_01485_amd as lg
from gpu_util import DEV, TOL_LSE, TOL_OUT, TOL_REL, assert_close, dq_delta_allowance, f32np
from oracle import lg_oracle as O

pytestmark = pytest.mark.gpu


def run_fwd_bwd(q, k, v, g, sink, window, block=1, stride=0, scale=0.0):
    qd, kd, vd, gd = (x.to(DEV) for x in (q, k, v, g))
    B, Hq, N, D = q.shape
    Hkv = k.shape[1]
    code = lg.LG_BF16 if q.dtype == torch.bfloat16 else lg.LG_F32
    out = torch.empty_like(qd)
    lse = torch.empty(B, Hq, N, dtype=torch.float32, device=DEV)
    lg.lg_sparse_attn_fwd(qd, kd, vd, out, lse, sink, window, block, stride, scale)
    need = lg.bwd_workspace_bytes(B, Hq, Hkv, N, D, sink, window, block, stride, code)
    assert need >= B * Hq * N * 4
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    dq = torch.full_like(qd, float("nan"))
    dk = torch.full_like(kd, float("nan"))
    dv = torch.full_like(vd, float("nan"))
    lg.lg_sparse_attn_bwd(qd, kd, vd, out, lse, gd, dq, dk, dv, ws, sink, window, block, stride, scale)
    torch.cuda.synchronize()
    return dq, dk, dv


def check_bwd(B, Hq, Hkv, N, D, sink, window, block=1, stride=0, dtype=torch.bfloat16, seed=1, q_mul=1.0,
              scale=0.0, by_tensor_max=False):
    q, k, v, g = lg_synth.prefill_inputs(B, Hq, Hkv, N, D, seed, dtype, with_dout=True, q_mul=q_mul)
    dq, dk, dv = run_fwd_bwd(q, k, v, g, sink, window, block, stride, scale)
    w = O.bwd(f32np(q), f32np(k), f32np(v), f32np(g), sink, window, block, stride, scale if scale > 0 else None)
    tag = "bwd B%d Hq%d Hkv%d N%d D%d s%d w%d b%d st%d %s" % (B, Hq, Hkv, N, D, sink, window, block, stride, dtype)
    allow = None
    if dtype == torch.bfloat16:  # Delta comes from the bf16-rounded forward output (see dq_delta_allowance)
        allow = dq_delta_allowance(f32np(q), f32np(k), f32np(g), w["out"], sink, window, block, stride,
                                   scale if scale > 0 else None)
    for name, got in (("dq", dq), ("dk", dk), ("dv", dv)):
        assert_close(f32np(got), w[name], TOL_OUT[dtype], TOL_REL[dtype], tag + " " + name, by_tensor_max,
                     allow=allow if name == "dq" else None)


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_sink_window_ragged_gqa(D, dtype):
    check_bwd(2, 4, 2, 700, D, 64, 200, dtype=dtype, seed=2)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("N,sink,window,block,stride", [
    (1, 0, 1, 1, 0), (33, 4, 8, 1, 0), (257, 0, 50, 1, 0), (500, 600, 3, 1, 0), (640, 5, 1000, 1, 0),
    (1024, 64, 192, 64, 8), (1000, 48, 96, 48, 3), (900, 0, 16, 16, 1), (777, 3, 10, 1, 7),
])
def test_patterns_and_edges(dtype, N, sink, window, block, stride):
    check_bwd(1, 2, 1, N, 128, sink, window, block, stride, dtype=dtype, seed=3)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_peaked_scores_and_custom_scale(dtype):
    check_bwd(1, 2, 2, 600, 128, 16, 100, dtype=dtype, seed=4, q_mul=4.0, by_tensor_max=True)
    check_bwd(1, 4, 1, 300, 64, 16, 100, dtype=dtype, seed=5, scale=0.3, by_tensor_max=True)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_masked_keys_get_exactly_zero_gradient(dtype):
    # upstream gradient only on a few rows: keys dead for all of them get dk = dv = 0 exactly,
    # and every other query row gets dq = 0 exactly
    N, D, sink, window = 1500, 128, 64, 256
    q, k, v, g = lg_synth.prefill_inputs(1, 2, 2, N, D, 7, dtype, with_dout=True)
    rows = np.arange(1300, 1400)
    g2 = torch.zeros_like(g)
    g2[:, :, rows] = g[:, :, rows]
    dq, dk, dv = run_fwd_bwd(q, k, v, g2, sink, window)
    m = O.mask(N, sink, window)
    dead = np.where(~m[rows].any(axis=0))[0]
    assert len(dead) > 1000
    assert (f32np(dk)[:, :, dead] == 0).all() and (f32np(dv)[:, :, dead] == 0).all()
    other = np.setdiff1d(np.arange(N), rows)
    assert (f32np(dq)[:, :, other] == 0).all()
    assert np.abs(f32np(dq)[:, :, rows]).sum() > 0


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("N,sink,window,block,stride", [(3000, 64, 512, 1, 0), (3000, 64, 192, 64, 8),
                                                        (2600, 0, 1100, 1, 0)])
def test_never_loaded_key_tiles_may_hold_nan_and_inf(dtype, N, sink, window, block, stride):
    """Key tiles that are dead for a whole 256-row query tile are never loaded by the forward and dq kernels
    (Section 3.2: a masked block is skipped by not loading it): NaN in K and Inf in V there leave out, lse and
    dq of those rows bit-identical.  (Rows outside the probed tile do see those keys and turn non-finite,
    and so do dk / dv of the poisoned keys themselves.)"""
    D = 128
    q, k, v, g = lg_synth.prefill_inputs(1, 2, 1, N, D, 71, dtype, with_dout=True)
    rows = np.arange(2048, 2304)                      # one 256-row query tile (a multiple of every kernel's tile)
    m = O.mask(N, sink, window, block, stride)
    tile_dead = ~m[rows].reshape(len(rows), -1)[:, :(N // 64) * 64].reshape(len(rows), N // 64, 64).any(axis=(0, 2))
    dead = np.where(np.repeat(tile_dead, 64))[0]      # every key of a 64-key tile no probed row sees
    assert len(dead) > 1000 and (dead < 2048).sum() > 500 and (dead >= 2304).sum() > 200
    k2, v2 = k.clone(), v.clone()
    k2[:, :, torch.as_tensor(dead)] = float("nan")
    v2[:, :, torch.as_tensor(dead)] = float("inf")
    g2 = torch.zeros_like(g)
    g2[:, :, rows] = g[:, :, rows]                    # upstream gradient on the probed rows only

    def run(kk, vv):
        qd, kd, vd, gd = (x.to(DEV) for x in (q, kk, vv, g2))
        out = torch.empty_like(qd)
        lse = torch.empty(1, 2, N, dtype=torch.float32, device=DEV)
        lg.lg_sparse_attn_fwd(qd, kd, vd, out, lse, sink, window, block, stride)
        code = lg.LG_BF16 if dtype == torch.bfloat16 else lg.LG_F32
        ws = torch.empty(lg.bwd_workspace_bytes(1, 2, 1, N, D, sink, window, block, stride, code), dtype=torch.uint8,
                         device=DEV)
        dq, dk, dv = torch.empty_like(qd), torch.empty_like(kd), torch.empty_like(vd)
        lg.lg_sparse_attn_bwd(qd, kd, vd, out, lse, gd, dq, dk, dv, ws, sink, window, block, stride)
        torch.cuda.synchronize()
        return out[:, :, rows].cpu(), lse[:, :, rows].cpu(), dq[:, :, rows].cpu()

    clean, poisoned = run(k, v), run(k2, v2)
    for name, a, b in zip(("out", "lse", "dq"), clean, poisoned):
        assert torch.isfinite(a.float()).all() and torch.equal(a, b), name
    w = O.bwd(f32np(q), f32np(k), f32np(v), f32np(g2), sink, window, block, stride, rows=(2048, 2304), keys=(0, 1))
    assert_close(f32np(poisoned[0]), w["out"][:, :, rows], TOL_OUT[dtype], TOL_REL[dtype], "poisoned out")
    al = dq_delta_allowance(f32np(q), f32np(k), f32np(g2), w["out"], sink, window, block, stride, rows=(2048, 2304))
    assert_close(f32np(poisoned[2]), w["dq"][:, :, rows], TOL_OUT[dtype], TOL_REL[dtype], "poisoned dq",
                 allow=al[:, :, rows] if dtype == torch.bfloat16 else None)


@pytest.mark.parametrize("B,Hq,Hkv,N,D,sink,window,block,stride", [
    # several column groups (sink + strided blocks), column parts longer than one chunk of 4096
    # rows, GQA, ragged ends; a virtual tile with fewer than 4 groups; token-granular strided columns
    (1, 4, 2, 9000, 128, 64, 128, 64, 4),
    (2, 2, 2, 5003, 64, 16, 48, 16, 3),
    (1, 2, 1, 4700, 128, 0, 64, 64, 16),
    (1, 2, 2, 4500, 128, 2, 6, 1, 9),
])
def test_strided_columns_long_context(B, Hq, Hkv, N, D, sink, window, block, stride):
    check_bwd(B, Hq, Hkv, N, D, sink, window, block, stride, dtype=torch.bfloat16, seed=41)


@pytest.mark.parametrize("B,Hq,Hkv,N,D,sink,window,block,stride", [
    # windows of 16 or more tiles at D = 128 select the kernels with 64 query rows / 64 keys per wave:
    # token-granular with a ragged end (sink tile handled by the main instance); GQA with batch
    # (column instance + partial sums folded into the main instance); block-granular; block-strided
    # (both instances in the 64-keys form); no sink and a window longer than most rows
    (1, 2, 2, 3001, 128, 64, 1024, 1, 0),
    (2, 4, 2, 2500, 128, 3, 900, 1, 0),
    (1, 2, 1, 3333, 128, 64, 1024, 64, 0),
    (1, 2, 2, 4100, 128, 64, 1024, 64, 8),
    (1, 1, 1, 2049, 128, 0, 2048, 1, 0),
    # column instance of the 64-keys-per-wave kernel: 29 column groups (a last virtual tile of one), column
    # parts longer than one chunk, GQA, ragged end
    (1, 4, 2, 9000, 128, 64, 1024, 64, 5),
])
def test_long_windows_wide_kernels(B, Hq, Hkv, N, D, sink, window, block, stride):
    check_bwd(B, Hq, Hkv, N, D, sink, window, block, stride, dtype=torch.bfloat16, seed=77)


def test_bwd_deterministic_long_window():
    q, k, v, g = lg_synth.prefill_inputs(1, 2, 2, 2000, 128, 10, torch.bfloat16, with_dout=True)
    a = run_fwd_bwd(q, k, v, g, 64, 1024)
    b = run_fwd_bwd(q, k, v, g, 64, 1024)
    for x, y in zip(a, b):
        assert torch.equal(x, y)


def test_bwd_deterministic():
    # sink + window without GQA has no atomics anywhere: bit-identical from run to run (the partial dk/dv
    # sums of column keys in strided or GQA calls are added with float atomics, in no fixed order)
    q, k, v, g = lg_synth.prefill_inputs(1, 4, 4, 900, 128, 9, torch.bfloat16, with_dout=True)
    a = run_fwd_bwd(q, k, v, g, 64, 300)
    b = run_fwd_bwd(q, k, v, g, 64, 300)
    for x, y in zip(a, b):
        assert torch.equal(x, y)


def test_config3_shape_reduced_n_all_heads():
    # config 3's heads, head dim, sink and window at a sequence the oracle finishes: N = 6144
    check_bwd(1, 32, 32, 6144, 128, 64, 4096, dtype=torch.bfloat16, seed=20241004)


def test_config3_full_size_sampled():
    """Training-step configuration as the benchmark launches it: B1, 32 heads, N=131072, D=128, sink 64,
    window 4096.  The oracle recomputes sampled query rows (dq) and sampled keys (dk, dv) of two heads."""
    B, H, N, D, sink, window = 1, 32, 131072, 128, 64, 4096
    q, k, v, g = lg_synth.prefill_inputs(B, H, H, N, D, 20241004, torch.bfloat16, with_dout=True, device=DEV)
    out = torch.empty_like(q)
    lse = torch.empty(B, H, N, dtype=torch.float32, device=DEV)
    lg.lg_sparse_attn_fwd(q, k, v, out, lse, sink, window)
    ws = torch.empty(lg.bwd_workspace_bytes(B, H, H, N, D, sink, window, 1, 0, lg.LG_BF16),
                     dtype=torch.uint8, device=DEV)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    lg.lg_sparse_attn_bwd(q, k, v, out, lse, g, dq, dk, dv, ws, sink, window)
    torch.cuda.synchronize()
    for t in (dq, dk, dv):
        assert torch.isfinite(t.float()).all()
    tol, rel = TOL_OUT[torch.bfloat16], TOL_REL[torch.bfloat16]
    for h, rows, keys in ((0, (0, 40), (0, 40)),                      # first rows; sink keys (seen by every row)
                          (0, (4080, 4120), (4140, 4180)),            # where the window starts to slide
                          (21, (70001, 70041), (99990, 100030)),      # steady state
                          (31, (N - 40, N), (N - 40, N))):            # ragged end of the sequence
        print("head", h, "rows", rows, "keys", keys, flush=True)
        a = [f32np(x[:, h:h + 1]) for x in (q, k, v, g)]
        w = O.bwd(*a, sink, window, rows=rows, keys=keys)
        al = dq_delta_allowance(a[0], a[1], a[3], w["out"], sink, window, rows=rows)
        assert_close(f32np(dq[0, h, rows[0]:rows[1]]), w["dq"][0, 0, rows[0]:rows[1]], tol, rel, "cfg3 dq h%d" % h,
                     allow=al[0, 0, rows[0]:rows[1]])
        assert_close(f32np(dk[0, h, keys[0]:keys[1]]), w["dk"][0, 0, keys[0]:keys[1]], tol, rel, "cfg3 dk h%d" % h)
        assert_close(f32np(dv[0, h, keys[0]:keys[1]]), w["dv"][0, 0, keys[0]:keys[1]], tol, rel, "cfg3 dv h%d" % h)
        assert_close(f32np(out[0, h, rows[0]:rows[1]]), w["out"][0, 0, rows[0]:rows[1]], tol, rel, "cfg3 out h%d" % h)
        assert_close(f32np(lse[0, h, rows[0]:rows[1]]), w["lse"][0, 0, rows[0]:rows[1]], TOL_LSE[torch.bfloat16], None,
                     "cfg3 lse h%d" % h)


def test_paper_block_settings_full_size_sampled():
    """Section 4.1 settings combined at the training length: 64-token blocks, 1 sink block, 32 local blocks
    and every 64th block as a strided column; B1, 32 heads, N=131072, D=128.  The oracle recomputes sampled
    query rows (dq) and sampled keys (dk, dv): sink keys, keys of a strided column (seen by every later row,
    accumulated over many workgroups), window-only keys, and the ragged end."""
    B, H, N, D, sink, window, block, stride = 1, 32, 131072, 128, 64, 2048, 64, 64
    q, k, v, g = lg_synth.prefill_inputs(B, H, H, N, D, 20241009, torch.bfloat16, with_dout=True, device=DEV)
    out = torch.empty_like(q)
    lse = torch.empty(B, H, N, dtype=torch.float32, device=DEV)
    lg.lg_sparse_attn_fwd(q, k, v, out, lse, sink, window, block, stride)
    ws = torch.empty(lg.bwd_workspace_bytes(B, H, H, N, D, sink, window, block, stride, lg.LG_BF16),
                     dtype=torch.uint8, device=DEV)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    lg.lg_sparse_attn_bwd(q, k, v, out, lse, g, dq, dk, dv, ws, sink, window, block, stride)
    torch.cuda.synchronize()
    for t in (dq, dk, dv):
        assert torch.isfinite(t.float()).all()
    tol, rel = TOL_OUT[torch.bfloat16], TOL_REL[torch.bfloat16]
    col = 63 * 64  # first strided column block
    for h, rows, keys in ((0, (0, 40), (20, 60)),                       # sink keys
                          (7, (70001, 70041), (col + 10, col + 50)),    # a strided column
                          (11, (120000, 120040), (1087 * 64 + 10, 1087 * 64 + 50)),   # a strided column past 64-key group 1024
                          (19, (100000, 100040), (90010, 90050)),       # window-only keys
                          (31, (N - 40, N), (N - 40, N))):              # the end of the sequence
        print("head", h, "rows", rows, "keys", keys, flush=True)
        a = [f32np(x[:, h:h + 1]) for x in (q, k, v, g)]
        w = O.bwd(*a, sink, window, block, stride, rows=rows, keys=keys)
        al = dq_delta_allowance(a[0], a[1], a[3], w["out"], sink, window, block, stride, rows=rows)
        assert_close(f32np(dq[0, h, rows[0]:rows[1]]), w["dq"][0, 0, rows[0]:rows[1]], tol, rel, "paper dq h%d" % h,
                     allow=al[0, 0, rows[0]:rows[1]])
        assert_close(f32np(dk[0, h, keys[0]:keys[1]]), w["dk"][0, 0, keys[0]:keys[1]], tol, rel, "paper dk h%d" % h)
        assert_close(f32np(dv[0, h, keys[0]:keys[1]]), w["dv"][0, 0, keys[0]:keys[1]], tol, rel, "paper dv h%d" % h)
        assert_close(f32np(out[0, h, rows[0]:rows[1]]), w["out"][0, 0, rows[0]:rows[1]], tol, rel, "paper out h%d" % h)
        assert_close(f32np(lse[0, h, rows[0]:rows[1]]), w["lse"][0, 0, rows[0]:rows[1]], TOL_LSE[torch.bfloat16], None,
                     "paper lse h%d" % h)


def test_one_million_tokens_sampled():
    """Index arithmetic at 2^20 tokens (8x the benchmark length), one head pair with GQA: forward and backward
    against the oracle on sampled rows and on sampled keys outside the sink (the sink keys would need the
    whole forward on the CPU)."""
    B, Hq, Hkv, N, D, sink, window = 1, 2, 1, 1 << 20, 128, 64, 4096
    q, k, v, g = lg_synth.prefill_inputs(B, Hq, Hkv, N, D, 20241010, torch.bfloat16, with_dout=True, device=DEV)
    out = torch.empty_like(q)
    lse = torch.empty(B, Hq, N, dtype=torch.float32, device=DEV)
    lg.lg_sparse_attn_fwd(q, k, v, out, lse, sink, window)
    ws = torch.empty(lg.bwd_workspace_bytes(B, Hq, Hkv, N, D, sink, window, 1, 0, lg.LG_BF16), dtype=torch.uint8,
                     device=DEV)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    lg.lg_sparse_attn_bwd(q, k, v, out, lse, g, dq, dk, dv, ws, sink, window)
    torch.cuda.synchronize()
    for t in (out, dq, dk, dv):
        assert torch.isfinite(t.float()).all()
    tol, rel = TOL_OUT[torch.bfloat16], TOL_REL[torch.bfloat16]
    a = [f32np(x) for x in (q, k, v, g)]
    for rows, keys in (((600001, 600041), (777770, 777810)), ((N - 40, N), (N - 40, N))):
        print("rows", rows, "keys", keys, flush=True)
        w = O.bwd(*a, sink, window, rows=rows, keys=keys)
        r, c = slice(*rows), slice(*keys)
        assert_close(f32np(out[0, :, r]), w["out"][0, :, r], tol, rel, "1M out")
        assert_close(f32np(lse[0, :, r]), w["lse"][0, :, r], TOL_LSE[torch.bfloat16], None, "1M lse")
        al = dq_delta_allowance(a[0], a[1], a[3], w["out"], sink, window, rows=rows)
        assert_close(f32np(dq[0, :, r]), w["dq"][0, :, r], tol, rel, "1M dq", allow=al[0, :, r])
        assert_close(f32np(dk[0, :, c]), w["dk"][0, :, c], tol, rel, "1M dk")
        assert_close(f32np(dv[0, :, c]), w["dv"][0, :, c], tol, rel, "1M dv")
