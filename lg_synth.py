"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

Holds no attention arithmetic: only a counter-based generator of i.i.d. N(0,1)
values (splitmix64-style integer mixing -> Box-Muller in float64), rounded to
float32 or bfloat16.  Element e of stream s under seed x depends only on
(x, s, e), so any slice of a tensor can be regenerated and the same bytes go
to the GPU path and to the CPU oracle.  The real workloads (Llama-2-7B/70B
activations at 128K tokens) need the paper's checkpoints and corpus, which are
not available; N(0,1) tensors of the same shapes stand in for them.
"""
import math

import torch

_M64 = (1 << 64) - 1
_GOLD = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB
STREAM_Q, STREAM_K, STREAM_V, STREAM_DOUT = 0, 1, 2, 3


def _s64(x):
    """Python int (mod 2^64) -> the int64 with the same bit pattern."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


def _mix_py(z):
    z &= _M64
    z = ((z ^ (z >> 30)) * _C1) & _M64
    z = ((z ^ (z >> 27)) * _C2) & _M64
    return z ^ (z >> 31)


def _lsr(x, n):
    """Logical right shift of an int64 tensor."""
    return (x >> n) & ((1 << (64 - n)) - 1)


def _mix(z):
    z = (z ^ _lsr(z, 30)) * _s64(_C1)
    z = (z ^ _lsr(z, 27)) * _s64(_C2)
    return z ^ _lsr(z, 31)


def _unit(bits):
    """int64 random bits -> float64 in (0, 1]."""
    return (_lsr(bits, 11).to(torch.float64) + 1.0) * (1.0 / 9007199254740992.0)


def normal_flat(n, seed, stream, start=0, device="cpu"):
    """float64 tensor of n standard normals: elements start .. start+n of (seed, stream).

    The arithmetic runs on `device`; the integer stream is identical everywhere, the
    float64 log/sin/cos may differ in the last place between devices, so a tensor
    that both the GPU path and the oracle consume is generated ONCE and copied."""
    base = _mix_py(_mix_py(seed * _GOLD + 0x632BE59BD9B4E019) ^ ((stream + 1) * 0xD1B54A32D192ED03))
    p0 = start // 2
    p1 = (start + n + 1) // 2
    out = torch.empty(2 * (p1 - p0), dtype=torch.float64, device=device)
    chunk = 1 << 22
    for a in range(p0, p1, chunk):
        b = min(a + chunk, p1)
        c = torch.arange(a, b, dtype=torch.int64, device=device)
        u1 = _unit(_mix(c * _s64(2 * _GOLD) + _s64(base + _GOLD)))
        u2 = _unit(_mix(c * _s64(2 * _GOLD) + _s64(base + 2 * _GOLD)))
        r = torch.sqrt(-2.0 * torch.log(u1))
        t = (2.0 * math.pi) * u2
        seg = out[2 * (a - p0): 2 * (b - p0)].view(-1, 2)
        seg[:, 0] = r * torch.cos(t)
        seg[:, 1] = r * torch.sin(t)
    off = start - 2 * p0
    return out[off: off + n]


def normal(shape, seed, stream, dtype=torch.float32, mul=1.0, device="cpu"):
    """Tensor of `shape` on `device`, values N(0,1)*mul rounded (nearest-even) to dtype."""
    n = 1
    for s in shape:
        n *= int(s)
    out = torch.empty(n, dtype=dtype, device=device)
    chunk = 1 << 24
    for a in range(0, n, chunk):
        m = min(chunk, n - a)
        z = normal_flat(m, seed, stream, start=a, device=device)
        if mul != 1.0:
            z = z * mul
        out[a: a + m] = z.to(torch.float32).to(dtype)
    return out.view(*shape)


def prefill_inputs(B, Hq, Hkv, N, D, seed, dtype=torch.float32, with_dout=False, q_mul=1.0, device="cpu"):
    """q [B,Hq,N,D], k,v [B,Hkv,N,D] (and dout [B,Hq,N,D]) ~ N(0,1)."""
    q = normal((B, Hq, N, D), seed, STREAM_Q, dtype, q_mul, device)
    k = normal((B, Hkv, N, D), seed, STREAM_K, dtype, 1.0, device)
    v = normal((B, Hkv, N, D), seed, STREAM_V, dtype, 1.0, device)
    if with_dout:
        return q, k, v, normal((B, Hq, N, D), seed, STREAM_DOUT, dtype, 1.0, device)
    return q, k, v


def decode_inputs(B, Hq, Hkv, C, D, seed, dtype=torch.float32, device="cpu"):
    """q [B,Hq,D] and cache contents k,v [B,Hkv,C,D] ~ N(0,1)."""
    q = normal((B, Hq, D), seed, STREAM_Q, dtype, 1.0, device)
    k = normal((B, Hkv, C, D), seed, STREAM_K, dtype, 1.0, device)
    v = normal((B, Hkv, C, D), seed, STREAM_V, dtype, 1.0, device)
    return q, k, v
