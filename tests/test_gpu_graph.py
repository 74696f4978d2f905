"""The entry points only enqueue kernels on the caller's stream (no allocation, no synchronisation,
no memset nodes), so a training step and a decode step can be captured into a HIP graph and replayed.
Every replay is checked against the eager result on the same inputs."""
import pytest
import torch

import lg_synth
import paper_2410_01485_amd as lg
from gpu_util import DEV

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("window,stride", [
    (128, 4),     # short window: the 8-wave backward kernels; column parts
    (1024, 8),    # long window at head dim 128: the 64-rows-per-wave backward kernels; column parts
])
def test_graph_replay_matches_eager(window, stride):
    B, Hq, Hkv, N, D, sink, block = 1, 4, 2, 5000, 128, 64, 64
    dt = torch.bfloat16
    q, k, v, g = (x.to(DEV) for x in lg_synth.prefill_inputs(B, Hq, Hkv, N, D, 71, dt, with_dout=True))
    out = torch.empty_like(q)
    lse = torch.empty(B, Hq, N, dtype=torch.float32, device=DEV)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    ws = torch.empty(lg.bwd_workspace_bytes(B, Hq, Hkv, N, D, sink, window, block, stride, lg.LG_BF16),
                     dtype=torch.uint8, device=DEV)
    slots = lg.lg_kv_cache_slots(N, sink, window, block, stride)
    kc = torch.zeros(B, Hkv, slots, D, dtype=dt, device=DEV)
    vc = torch.zeros_like(kc)
    q1 = torch.empty(B, Hq, D, dtype=dt, device=DEV)
    o1 = torch.empty_like(q1)
    l1 = torch.empty(B, Hq, dtype=torch.float32, device=DEV)
    dws = torch.empty(max(16, lg.decode_cache_workspace_bytes(B, Hq, Hkv, N, D, sink, window, block, stride,
                                                              lg.LG_BF16)), dtype=torch.uint8, device=DEV)

    def step():
        lg.lg_sparse_attn_fwd(q, k, v, out, lse, sink, window, block, stride)
        lg.lg_sparse_attn_bwd(q, k, v, out, lse, g, dq, dk, dv, ws, sink, window, block, stride)
        lg.lg_kv_ring_append(k, v, kc, vc, 0, sink, window, block, stride)
        q1.copy_(q[:, :, N - 1])
        lg.lg_sparse_attn_decode_cache(q1, kc, vc, o1, l1, dws, N, sink, window, block, stride)

    step()  # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        fresh = [x.to(DEV) for x in lg_synth.prefill_inputs(B, Hq, Hkv, N, D, 80 + rep, dt, with_dout=True)]
        for dst, src in zip((q, k, v, g), fresh):
            dst.copy_(src)
        for t in (out, dq, dk, dv, o1):
            t.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (out, lse, dq, dk, dv, o1, l1)]
        step()  # eager, same inputs
        torch.cuda.synchronize()
        for name, a, b in zip(("out", "lse", "dq", "dk", "dv", "decode out", "decode lse"), got,
                              (out, lse, dq, dk, dv, o1, l1)):
            if name in ("dk", "dv"):   # column keys are summed with float atomics: order-dependent last bits
                assert torch.allclose(a.float(), b.float(), rtol=2e-2, atol=2e-2), (rep, name)
            else:
                assert torch.equal(a, b), (rep, name)
