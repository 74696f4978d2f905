"""Run one entry point on one benchmark workload a few times, for rocprofv3.

    rocprofv3 --kernel-trace --stats --output-format csv -d OUT -o NAME -- \
        python3 paper_2410_01485_amd/prof_run.py {fwd|bwd|bwd_strided|decode|fwd_strided|fwd_gqa|copy} [reps]

fwd / bwd   : B1 H32 D128 N131072 bf16, sink 64 + window 4096 (the training-step workload)
bwd_strided : B1 H32 D128 N131072 bf16, 64-token blocks: sink block, window 2048, every 64th block
fwd_strided : B1 H32 D128 N32768 bf16, 64-token blocks: own + 2 preceding, sink block, every 8th
fwd_gqa     : B1 Hq64/Hkv8 D128 N131072 bf16, sink 64 + window 4096
decode      : B16 H32 D128 bf16, 64 + 4096 cache slots, three rotating cache sets
copy        : a plain elementwise pass over 1 GiB (reads 2^30 bytes, writes 2^30 bytes): the yardstick
              that FETCH_SIZE / WRITE_SIZE counter readings are scaled by
Inputs are filled on the device (values do not matter to a profile).
"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def main():
    import torch

    import paper_2410_01485_amd as lg

    what = sys.argv[1]
    reps = int(sys.argv[2]) if len(sys.argv) > 2 else 3
    dev = "cuda:0"
    bf = torch.bfloat16

    def rnd(*shape):
        return torch.empty(*shape, device=dev, dtype=torch.float32).normal_().to(bf)

    if what == "copy":
        a = torch.empty(1 << 28, dtype=torch.float32, device=dev).zero_()
        b = torch.empty_like(a)
        for _ in range(reps):
            torch.add(a, 1.0, out=b)   # an elementwise kernel: reads 2^30 bytes, writes 2^30 bytes
    elif what in ("fwd", "bwd", "bwd_strided", "fwd_strided", "fwd_gqa"):
        Hq, Hkv, N, sink, window, block, stride = 32, 32, 131072, 64, 4096, 1, 0
        if what == "fwd_strided":
            N, sink, window, block, stride = 32768, 64, 192, 64, 8
        if what == "fwd_gqa":
            Hq, Hkv = 64, 8
        if what == "bwd_strided":
            sink, window, block, stride = 64, 2048, 64, 64
        D = 128
        q, k, v = rnd(1, Hq, N, D), rnd(1, Hkv, N, D), rnd(1, Hkv, N, D)
        out = torch.empty_like(q)
        lse = torch.empty(1, Hq, N, dtype=torch.float32, device=dev)
        lg.lg_sparse_attn_fwd(q, k, v, out, lse, sink, window, block, stride)
        if what in ("bwd", "bwd_strided"):
            g = rnd(1, Hq, N, D)
            ws = torch.empty(lg.bwd_workspace_bytes(1, Hq, Hkv, N, D, sink, window, block, stride, lg.LG_BF16),
                             dtype=torch.uint8, device=dev)
            dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
            for _ in range(reps):
                lg.lg_sparse_attn_bwd(q, k, v, out, lse, g, dq, dk, dv, ws, sink, window, block, stride)
        else:
            for _ in range(reps):
                lg.lg_sparse_attn_fwd(q, k, v, out, lse, sink, window, block, stride)
    elif what == "decode":
        B, H, D, sink, window, N = 16, 32, 128, 64, 4096, 131072
        C = sink + window
        sets = [(rnd(B, H, C, D), rnd(B, H, C, D)) for _ in range(3)]
        q = rnd(B, H, D)
        out = torch.empty_like(q)
        lse = torch.empty(B, H, dtype=torch.float32, device=dev)
        need = lg.decode_workspace_bytes(B, H, H, N, D, sink, window, lg.LG_BF16)
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
        for i in range(3 * reps):
            kc, vc = sets[i % 3]
            lg.lg_sparse_attn_decode(q, kc, vc, out, lse, ws, N, sink, window)
    else:
        sys.exit("unknown workload " + what)
    torch.cuda.synchronize()


if __name__ == "__main__":
    main()
