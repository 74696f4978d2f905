#!/usr/bin/env python3
"""Benchmark of the sparse-attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One step = the training pass of one sparse layer on the Llama-2-7B-shaped 128K workload
(B1, 32 heads, D128, N131072, bf16, sink 64 + window 4096): forward (out, lse) followed by
backward (dq kernel, which also forms Delta, and dk/dv kernel), inputs resident in HBM.  The headline
value is effective TFLOP/s: algorithmic flops of the live (query, key) pairs (4*D forward,
10*D backward per pair per head) divided by the measured step time.  The same run also times
decode over the 64+4096-slot ring cache (B16, 32 heads), the other workloads of the benchmark set
(float32 correctness config, block-strided forward at 32K, GQA forward at 128K), the paper's block-granular
settings, a 32-layer attention-only stack (12 full + 20 sparse layers, executed call by call) against 32 full
layers, and the fp64 CPU oracle on a bounded sample.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

# HBM-side bytes per launch on these two workloads (read, written), from the rocprofv3
# FETCH_SIZE / WRITE_SIZE passes summarised in profiles/hbm_traffic_fwd_bwd_decode.txt, each
# scaled by what the same counter reads for a copy kernel of known size.  Counter runs are
# separate from timed runs, so these are constants here, not measured by this script.
MEASURED_HBM_BYTES = {
    "fwd_bf16_kernel": (4.25e9, 1.090e9),
    "dq_wide_bf16_kernel": (6.57e9, 1.110e9),
    "dkdv_wide_bf16_kernel": (7.85e9, 2.160e9),
    "decode_kernel": (1.09e9, 0.000e9),
}


def live_pairs(N, sink, window):
    """Token-level live (i, j) pairs of the sink + window mask (closed form per row)."""
    return sum(min(i + 1, window) + min(sink, max(0, i - window + 1)) for i in range(N))


def block_pairs(N, sink, window, block, stride):
    """Live (i, j) pairs of a block-granular pattern: per query block, the live key blocks below the
    diagonal are whole, the diagonal block is causal."""
    nb, sb, wb, tot = (N + block - 1) // block, sink // block, window // block, 0
    for qb in range(nb):
        rows = min(block, N - qb * block)
        below = set(range(min(sb, qb))) | set(range(max(0, qb - wb + 1), qb))
        if stride > 0:
            below |= set(range(stride - 1, qb, stride))
        tot += len(below) * rows * block + rows * (rows + 1) // 2
    return tot


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the headline workloads (training step, decode): what the kernel-trace profile runs")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on ONE GPU (every (batch, head) is independent, so more GPUs "
                 "would only shard heads with no exchange); run with --gpus 1")

    import torch

    import lg_synth
    import paper_2410_01485_amd as lg

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    lg.lib()  # fails loudly if the HIP library is not built
    dev = "cuda:0"
    K, W = args.steps, args.warmup

    # ------------------------------------------------------------------ training step, 128K
    B, H, N, D, sink, window = 1, 32, 131072, 128, 64, 4096
    q, k, v, g = lg_synth.prefill_inputs(B, H, H, N, D, 20241004, torch.bfloat16, with_dout=True, device=dev)
    out = torch.empty_like(q)
    lse = torch.empty(B, H, N, dtype=torch.float32, device=dev)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    ws = torch.empty(lg.bwd_workspace_bytes(B, H, H, N, D, sink, window, 1, 0, lg.LG_BF16),
                     dtype=torch.uint8, device=dev)

    def step():
        lg.lg_sparse_attn_fwd(q, k, v, out, lse, sink, window)
        lg.lg_sparse_attn_bwd(q, k, v, out, lse, g, dq, dk, dv, ws, sink, window)

    for _ in range(W):
        step()
    torch.cuda.synchronize()
    # The timed region: K steps through the product entry points (lg_sparse_attn_fwd, lg_sparse_attn_bwd),
    # bracketed by events on the stream the binding hands to the library (torch's current stream).
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(K)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(K):
        ev[s][0].record()
        lg.lg_sparse_attn_fwd(q, k, v, out, lse, sink, window)
        ev[s][1].record()
        lg.lg_sparse_attn_bwd(q, k, v, out, lse, g, dq, dk, dv, ws, sink, window)
        ev[s][2].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / K
    fwd_ms = sum(e[0].elapsed_time(e[1]) for e in ev) / K
    bwd_ms = sum(e[1].elapsed_time(e[2]) for e in ev) / K
    step_ms = ev[0][0].elapsed_time(ev[-1][2]) / K
    per_step = sorted(e[0].elapsed_time(e[2]) for e in ev)
    # The split of the backward over its kernels: a separate, untimed pass of K calls of the library's timing
    # variant of the same entry point (identical launches, each kernel bracketed by HIP events on the launch
    # stream; it synchronises after every call, which is why it is not what the timed region runs).
    split = [0.0, 0.0, 0.0]
    for _ in range(K):
        ms = lg.lg_debug_bwd_kernel_ms(q, k, v, out, lse, g, dq, dk, dv, ws, sink, window)
        split = [a + b / K for a, b in zip(split, ms)]

    pairs = live_pairs(N, sink, window) * H * B
    fl_fwd, fl_bwd = 4.0 * D * pairs, 10.0 * D * pairs
    value = (fl_fwd + fl_bwd) / (step_ms * 1e-3) / 1e12
    # algorithmic flops per kernel: forward S,PV (4D); dq kernel S,dP,dQ (6D); dk/dv kernel dV,dK (4D; its
    # recomputation of S and dP is not counted)
    kernels = [
        {"kernel": "fwd_bf16_kernel", "ms": fwd_ms, "flops": fl_fwd},
        # (head dim 128 with a window of 16+ tiles: the library picks its 64-rows-per-wave kernels)
        {"kernel": "dq_wide_bf16_kernel", "ms": split[1], "flops": 6.0 * D * pairs},
        {"kernel": "dkdv_wide_bf16_kernel", "ms": split[2], "flops": 4.0 * D * pairs},
    ]
    for kk in kernels:
        kk["tflops"] = kk["flops"] / (kk["ms"] * 1e-3) / 1e12
        kk["frac"] = kk["tflops"] / PEAK_BF16_TFLOPS
    dom = max(kernels, key=lambda x: x["ms"])
    roofline = {"bound": "mfma", "kernel": dom["kernel"], "achieved": dom["tflops"], "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": dom["frac"], "traffic": sum(MEASURED_HBM_BYTES[dom["kernel"]]),
                "avg_launch_ms": dom["ms"],
                "kernels": [{"kernel": x["kernel"], "ms": round(x["ms"], 4), "tflops": round(x["tflops"], 1),
                             "frac": round(x["frac"], 4)} for x in kernels],
                "bwd_setup_ms": round(split[0], 4),  # clearing the work-queue counters (Delta is formed in the dq kernel)
                "fwd": {"ms": round(fwd_ms, 4), "tflops": round(fl_fwd / fwd_ms / 1e9, 1),
                        "frac": round(fl_fwd / fwd_ms / 1e9 / PEAK_BF16_TFLOPS, 4)},
                "bwd": {"ms": round(bwd_ms, 4), "tflops": round(fl_bwd / bwd_ms / 1e9, 1),
                        "frac": round(fl_bwd / bwd_ms / 1e9 / PEAK_BF16_TFLOPS, 4)}}
    # the paper's own block-granular settings (Section 4.1) on the same tensors, 3 launches each:
    # attention sink (1 sink block + 32 local blocks) and sink + local + every 64th block
    paper = []
    for name, (ps, pw, pb, pst) in (() if args.no_extras else
                                    (("attn_sink b64: sink 64, window 2048", (64, 2048, 64, 0)),
                                     ("block_sparse b64: sink 64, window 2048, stride 64", (64, 2048, 64, 64)))):
        pws = torch.empty(lg.bwd_workspace_bytes(B, H, H, N, D, ps, pw, pb, pst, lg.LG_BF16),
                          dtype=torch.uint8, device=dev)
        pp = block_pairs(N, ps, pw, pb, pst) * H * B
        lg.lg_sparse_attn_fwd(q, k, v, out, lse, ps, pw, pb, pst)
        lg.lg_sparse_attn_bwd(q, k, v, out, lse, g, dq, dk, dv, pws, ps, pw, pb, pst)
        torch.cuda.synchronize()
        e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        f_ms = b_ms = 0.0
        for _ in range(3):
            e0.record()
            lg.lg_sparse_attn_fwd(q, k, v, out, lse, ps, pw, pb, pst)
            e1.record()
            lg.lg_sparse_attn_bwd(q, k, v, out, lse, g, dq, dk, dv, pws, ps, pw, pb, pst)
            e2.record()
            torch.cuda.synchronize()
            f_ms += e0.elapsed_time(e1) / 3
            b_ms += e1.elapsed_time(e2) / 3
        paper.append({"pattern": name, "live_pairs_per_head": pp // (H * B), "fwd_ms": round(f_ms, 3),
                      "bwd_ms": round(b_ms, 3),
                      "tflops": round(14.0 * D * pp / ((f_ms + b_ms) * 1e-3) / 1e12, 1),
                      "frac": round(14.0 * D * pp / ((f_ms + b_ms) * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)})
        del pws
    # Full causal attention through the same kernels (window >= N) and the paper's hybrid as an executed
    # attention-only stack (Section 3.1: 32 layers, sparse attention in the bottom 10 and top 10 layers, full
    # attention in the middle 12): 32 consecutive layer calls on one stream, each layer's output feeding the
    # next layer's queries (forward) and each layer's dq feeding the layer below as its upstream gradient
    # (backward, reverse order), timed end to end, beside the same stack with 32 full layers.
    full = None
    if not args.no_extras:
        L_ALL = 32
        hybrid = [i < 10 or i >= 22 for i in range(L_ALL)]          # True = sparse layer
        fws = torch.empty(lg.bwd_workspace_bytes(B, H, H, N, D, 0, N, 1, 0, lg.LG_BF16), dtype=torch.uint8,
                          device=dev)
        # per-layer activations kept for the backward: queries (= the previous layer's out), out, lse
        acts = [q] + [torch.empty_like(q) for _ in range(L_ALL)]
        lses = [torch.empty_like(lse) for _ in range(L_ALL)]
        grads = [torch.empty_like(q), torch.empty_like(q)]

        def stack_fwd(sparse_layers):
            for i in range(L_ALL):
                sk_, w_ = (sink, window) if sparse_layers[i] else (0, N)
                lg.lg_sparse_attn_fwd(acts[i], k, v, acts[i + 1], lses[i], sk_, w_)

        def stack_bwd(sparse_layers):
            gin = g
            for i in reversed(range(L_ALL)):
                sk_, w_ = (sink, window) if sparse_layers[i] else (0, N)
                gout = grads[i & 1]
                lg.lg_sparse_attn_bwd(acts[i], k, v, acts[i + 1], lses[i], gin, gout, dk, dv,
                                      ws if sparse_layers[i] else fws, sk_, w_)
                gin = gout

        def timed(fn, *a):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            fn(*a)
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1)

        # warm-up: one full-causal layer forward and backward (the sparse kernels ran above)
        lg.lg_sparse_attn_fwd(q, k, v, out, lse, 0, N)
        lg.lg_sparse_attn_bwd(q, k, v, out, lse, g, dq, dk, dv, fws, 0, N)
        cf = timed(lg.lg_sparse_attn_fwd, q, k, v, out, lse, 0, N)
        cb = timed(lg.lg_sparse_attn_bwd, q, k, v, out, lse, g, dq, dk, dv, fws, 0, N)
        all_full = [False] * L_ALL
        hyb_fwd = timed(stack_fwd, hybrid)
        hyb_bwd = timed(stack_bwd, hybrid)
        ful_fwd = timed(stack_fwd, all_full)
        ful_bwd = timed(stack_bwd, all_full)
        cpairs = N * (N + 1) // 2 * H * B
        full = {"workload": "full causal attention, same shape (window = N), one layer",
                "fwd_ms": round(cf, 2), "bwd_ms": round(cb, 2),
                "tflops": round(14.0 * D * cpairs / ((cf + cb) * 1e-3) / 1e12, 1),
                "frac": round(14.0 * D * cpairs / ((cf + cb) * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                "stack_32_layers_executed": {
                    "what": "attention-only stack, 32 consecutive layer calls per pass on one stream: hybrid = 10 "
                            "sparse + 12 full + 10 sparse layers (sink 64 + window 4096), against 32 full layers; "
                            "the paper's end-to-end figures (1.55x training, 1.67x prefill, whole model, A100s) "
                            "include the linear layers and are context only",
                    "hybrid_prefill_ms": round(hyb_fwd, 1), "all_full_prefill_ms": round(ful_fwd, 1),
                    "hybrid_train_ms": round(hyb_fwd + hyb_bwd, 1), "all_full_train_ms": round(ful_fwd + ful_bwd, 1),
                    "attention_speedup_prefill": round(ful_fwd / hyb_fwd, 2),
                    "attention_speedup_train": round((ful_fwd + ful_bwd) / (hyb_fwd + hyb_bwd), 2)}}
        del fws, acts, lses, grads
    del q, k, v, g, out, lse, dq, dk, dv, ws
    torch.cuda.empty_cache()

    # ------------------------------------------------------------------ the other workloads of the benchmark set
    # (forward only, as their definitions say): the float32 correctness config, the block-strided forward at
    # 32K and the GQA forward at 128K.  5 launches each after 2 warm-ups, events around the product call.
    PEAK_F32_VECTOR_TFLOPS = 157.3
    others = []
    if not args.no_extras:
        def fwd_config(name, what, Bc, Hq, Hkv, Nc, Dc, dt, sk_, w_, blk, st_, seed, pairs_per_head, extra):
            cq, ck, cv = lg_synth.prefill_inputs(Bc, Hq, Hkv, Nc, Dc, seed, dt, device=dev)
            co = torch.empty_like(cq)
            cl = torch.empty(Bc, Hq, Nc, dtype=torch.float32, device=dev)
            for _ in range(2):
                lg.lg_sparse_attn_fwd(cq, ck, cv, co, cl, sk_, w_, blk, st_)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(5):
                lg.lg_sparse_attn_fwd(cq, ck, cv, co, cl, sk_, w_, blk, st_)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 5
            fl = 4.0 * Dc * pairs_per_head * Hq * Bc
            peak = PEAK_BF16_TFLOPS if dt == torch.bfloat16 else PEAK_F32_VECTOR_TFLOPS
            rec = {"config": name, "workload": what, "fwd_ms": round(ms, 4), "flops": fl,
                   "tflops": round(fl / (ms * 1e-3) / 1e12, 3), "peak_tflops": peak,
                   "frac": round(fl / (ms * 1e-3) / 1e12 / peak, 4), "live_pairs_per_head": pairs_per_head}
            rec.update(extra)
            others.append(rec)

        fwd_config("config 1", "B1 H1 N1024 D64 float32, sink 16 + window 128 (correctness config: one small "
                   "launch, latency-bound; priced against the float32 vector peak)", 1, 1, 1, 1024, 64,
                   torch.float32, 16, 128, 1, 0, 20241002, live_pairs(1024, 16, 128), {"bound": "alu"})
        nblk = 32768 // 64
        live_blocks = sum(len(set(range(min(1, qb))) | set(range(max(0, qb - 2), qb + 1)) | set(range(7, qb, 8)))
                          for qb in range(nblk))
        fwd_config("config 2", "B1 H32/32 N32768 D128 bf16, 64-token blocks: own block + 2 preceding, sink block, "
                   "every 8th earlier block", 1, 32, 32, 32768, 128, torch.bfloat16, 64, 192, 64, 8, 20241003,
                   block_pairs(32768, 64, 192, 64, 8),
                   {"bound": "mfma", "live_blocks_per_head": live_blocks, "causal_blocks_per_head": nblk * (nblk + 1) // 2})
        fwd_config("config 4", "B1 Hq64/Hkv8 (GQA) N131072 D128 bf16, sink 64 + window 4096", 1, 64, 8, 131072, 128,
                   torch.bfloat16, 64, 4096, 1, 0, 20241005, live_pairs(131072, 64, 4096), {"bound": "mfma"})
        torch.cuda.empty_cache()

    # ------------------------------------------------------------------ prefill of a batch of different lengths
    # (the serving setting): requests packed per head, one forward call, beside the same requests padded to
    # the longest in a [requests, H, longest, D] batch.  Two mixes: eight long requests (2K .. 64K tokens) and
    # 256 short ones (256 .. 2048 tokens, seeded).
    varlen = None
    if not args.no_extras:
        import numpy as np

        def timed_ms(fn, reps=5):
            for _ in range(2):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps

        def varlen_case(what, lens, seed):
            cu = [0]
            for n in lens:
                cu.append(cu[-1] + n)
            T = cu[-1]
            vq, vk, vv = (t[0] for t in lg_synth.prefill_inputs(1, H, H, T, D, seed, torch.bfloat16, device=dev))
            vo = torch.empty_like(vq)
            vl = torch.empty(H, T, dtype=torch.float32, device=dev)
            pq, pk, pv = lg_synth.prefill_inputs(len(lens), H, H, max(lens), D, seed + 1, torch.bfloat16, device=dev)
            po = torch.empty_like(pq)
            pl = torch.empty(len(lens), H, max(lens), dtype=torch.float32, device=dev)
            v_ms = timed_ms(lambda: lg.lg_sparse_attn_fwd_varlen(vq, vk, vv, vo, vl, cu, sink, window))
            p_ms = timed_ms(lambda: lg.lg_sparse_attn_fwd(pq, pk, pv, po, pl, sink, window))
            vfl = 4.0 * D * H * sum(live_pairs(n, sink, window) for n in lens)
            rec = {"workload": "prefill forward of %s, H32/32 D128 bf16, sink 64 + window 4096, packed per head "
                               "(lg_sparse_attn_fwd_varlen)" % what,
                   "requests": len(lens), "tokens": T, "fwd_ms": round(v_ms, 3), "flops": vfl,
                   "tflops": round(vfl / (v_ms * 1e-3) / 1e12, 1),
                   "frac": round(vfl / (v_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                   "padded_batch_fwd_ms": round(p_ms, 3), "padded_tokens": len(lens) * max(lens),
                   "speedup_vs_padded": round(p_ms / v_ms, 2)}
            del vq, vk, vv, vo, vl, pq, pk, pv, po, pl
            torch.cuda.empty_cache()
            return rec

        long_mix = [2048, 4096, 8192, 12288, 16384, 24576, 32768, 65536]
        short_mix = [int(x) for x in np.random.default_rng(20241014).integers(256, 2049, 256)]
        varlen = [varlen_case("8 requests of %s tokens" % long_mix, long_mix, 20241012),
                  varlen_case("256 requests of 256 .. 2048 tokens (seeded, %d in all)" % sum(short_mix), short_mix,
                              20241015)]

    # ------------------------------------------------------------------ decode, ring cache
    dB, dH, dsink, dwin, dN = 16, 32, 64, 4096, 131072
    C = dsink + dwin
    sets = []
    for r in range(3):  # rotate > 256 MB of distinct caches so no launch re-reads a cached one
        dq_, kc, vc = lg_synth.decode_inputs(dB, dH, dH, C, D, 20241006 + r, torch.bfloat16, device=dev)
        sets.append((dq_, kc, vc))
    dout = torch.empty_like(sets[0][0])
    dlse = torch.empty(dB, dH, dtype=torch.float32, device=dev)
    need = lg.decode_workspace_bytes(dB, dH, dH, dN, D, dsink, dwin, lg.LG_BF16)
    dws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    it = [0]

    def dstep():
        a, b_, c_ = sets[it[0] % 3]
        it[0] += 1
        lg.lg_sparse_attn_decode(a, b_, c_, dout, dlse, dws, dN, dsink, dwin)

    for _ in range(max(W, 10)):  # the memory clock needs a few launches to settle after the prefill part
        dstep()
    torch.cuda.synchronize()
    reps = max(K * 5, 30)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        dstep()
    e1.record()
    torch.cuda.synchronize()
    dec_ms = e0.elapsed_time(e1) / reps
    dec_bytes = 2.0 * dB * dH * C * D * 2 + 2.0 * dB * dH * D * 2
    dec_gbs = dec_bytes / (dec_ms * 1e-3) / 1e9
    decode = {"workload": "B16 H32 D128 bf16, ring cache 64 sink + 4096 window slots, context 131072",
              "us_per_call": round(dec_ms * 1e3, 2), "bytes": dec_bytes,
              "roofline": {"bound": "hbm", "achieved": round(dec_gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                           "frac": round(dec_gbs / PEAK_HBM_GBS, 4),
                           "traffic": sum(MEASURED_HBM_BYTES["decode_kernel"])}}

    # (extras) A/B: the paper's decode design, work split over the head dimension instead of the slots
    if not args.no_extras:
        for _ in range(3):
            a, b_, c_ = sets[it[0] % 3]
            it[0] += 1
            sd_ws = lg.lg_debug_decode_split_headdim(a, b_, c_, dout, dlse, dN, dsink, dwin)
        e0.record()
        for _ in range(reps):
            a, b_, c_ = sets[it[0] % 3]
            it[0] += 1
            lg.lg_debug_decode_split_headdim(a, b_, c_, dout, dlse, dN, dsink, dwin)
        e1.record()
        torch.cuda.synchronize()
        sd_ms = e0.elapsed_time(e1) / reps
        decode["split_head_dim_variant"] = {
            "what": "same workload, head dimension split in 2 across workgroups (two passes, partial scores "
                    "through a workspace); includes the workspace allocation of the Python helper",
            "us_per_call": round(sd_ms * 1e3, 2), "gbs": round(dec_bytes / (sd_ms * 1e-3) / 1e9, 1)}
        del sd_ws

    # (extras) the block-sparse + sink + window pattern of Section 4.1 over the same cache tensors:
    # 64-token blocks, 1 sink block, 32 local blocks, one retained block per 64 (4160 slots too)
    pb, ps, pwin, pstr = 64, 64, 2048, 64
    assert lg.lg_kv_cache_slots(dN, ps, pwin, pb, pstr) == C
    keys = sum(n for _, n in lg.lg_debug_decode_segments(dN, ps, pwin, pb, pstr))
    need = lg.decode_cache_workspace_bytes(dB, dH, dH, dN, D, ps, pwin, pb, pstr, lg.LG_BF16)
    pws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)

    def pstep():
        a, b_, c_ = sets[it[0] % 3]
        it[0] += 1
        lg.lg_sparse_attn_decode_cache(a, b_, c_, dout, dlse, pws, dN, ps, pwin, pb, pstr)

    for _ in range(3):
        pstep()
    e0.record()
    for _ in range(reps):
        pstep()
    e1.record()
    torch.cuda.synchronize()
    p_ms = e0.elapsed_time(e1) / reps
    p_bytes = 2.0 * dB * dH * keys * D * 2 + 2.0 * dB * dH * D * 2
    decode["block_sparse"] = {"workload": "same caches, block 64: 1 sink block + 32 local blocks + every 64th "
                                          "block (%d of %d slots live)" % (keys, C),
                              "us_per_call": round(p_ms * 1e3, 2), "bytes": p_bytes,
                              "gbs": round(p_bytes / (p_ms * 1e-3) / 1e9, 1),
                              "frac": round(p_bytes / (p_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}

    # ------------------------------------------------------------------ CPU oracle baseline
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import lg_oracle as O
        sN = N  # one of the 32 heads at the full length: about 1/32 of a step
        sq, sk, sv, sg = (x.float().numpy() for x in
                          lg_synth.prefill_inputs(1, 1, 1, sN, D, 20241004, torch.bfloat16, with_dout=True))
        t0 = time.perf_counter()
        O.bwd(sq, sk, sv, sg, sink, window)   # fp64 forward + backward
        dt = time.perf_counter() - t0
        sp = live_pairs(sN, sink, window)
        cpu = {"value": 14.0 * D * sp / dt / 1e12, "unit": "TFLOP/s", "cores": O.threads(), "kind": "oracle",
               "sample": "fp64 oracle forward+backward of 1 of the 32 heads at N=131072 (sink 64, window "
                         "4096): %.1f s; a whole step would take 32x that" % dt}

    print(json.dumps({
        "metric": "sparse-attn fwd+bwd ms & TFLOP/s @128K; decode GB/s vs HBM peak (1 GPU)",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": step_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "Llama-2-7B-shaped training step of one sparse layer: causal sink+window "
                               "attention fwd+bwd, B1 H32/32 D128 N131072 bf16, sink 64, window 4096",
                   "target": "50 % of the bf16 MFMA peak for prefill forward and backward, 70 % of the HBM peak "
                             "for decode",
                   "target_met": {"prefill_fwd": bool(fl_fwd / fwd_ms / 1e9 / PEAK_BF16_TFLOPS >= 0.5),
                                  "prefill_bwd": bool(fl_bwd / bwd_ms / 1e9 / PEAK_BF16_TFLOPS >= 0.5),
                                  "decode": bool(dec_gbs / PEAK_HBM_GBS >= 0.7)},
                   "live_pairs_per_head": pairs // (H * B), "flops_per_step": fl_fwd + fl_bwd,
                   "wall_ms_per_step": round(wall_ms, 3),
                   "ms_per_step_median": round(per_step[len(per_step) // 2], 3),
                   "ms_per_step_min": round(per_step[0], 3)},
        "roofline": roofline, "cpu_baseline": cpu, "decode": decode, "other_configs": others,
        "paper_block_settings": paper, "full_causal": full, "varlen_prefill": varlen,
    }))


if __name__ == "__main__":
    main()
