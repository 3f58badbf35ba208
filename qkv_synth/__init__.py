"""Seeded synthetic inputs: K/V caches, token scores and bit-width vectors.

Stand-ins for real Llama-3.1-8B caches (weights are not available): the shapes and value
structure follow the benchmark configurations (outlier key channels, per-token value
scale).  This module serves both the CPU oracle's tests and the GPU path and holds
none of the method's arithmetic: it only draws numbers.

The generator is counter based: value i of stream s under seed k is a pure function
hash(k, s, i), evaluated with wrapping int64 tensor arithmetic, so the integer draws are
identical on every device and any sub-range can be regenerated alone.
"""
import math

import torch

_M1 = -4658895280553007687   # 0xBF58476D1CE4E5B9 as int64
_M2 = -7723592293110705685   # 0x94D049BB133111EB as int64
_GOLD = -7046029254386353131  # 0x9E3779B97F4A7C15 as int64


def _lsr(x, s):
    """Logical shift right of int64 tensors."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix64(x):
    x = (x ^ _lsr(x, 30)) * _M1
    x = (x ^ _lsr(x, 27)) * _M2
    return x ^ _lsr(x, 31)


def _wrap64(v):
    v &= (1 << 64) - 1
    return v - (1 << 64) if v >= (1 << 63) else v


def _key(seed, stream):
    """Scalar key for (seed, stream): one mix round in Python integers, wrapped to int64."""
    x = (seed * 0x9E3779B97F4A7C15 + stream * 0xD1B54A32D192ED03 + 0x2545F4914F6CDD1D) & ((1 << 64) - 1)
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & ((1 << 64) - 1)
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & ((1 << 64) - 1)
    x ^= x >> 31
    return _wrap64(x)


def raw_u64(seed, stream, start, count, device="cpu"):
    """int64 tensor of `count` hashed draws for counters start .. start+count-1."""
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    return _mix64(idx * _GOLD + _key(seed, stream))


def uniform01(seed, stream, start, count, device="cpu"):
    """float32 uniforms strictly inside (0, 1), 24 bits each."""
    r = _lsr(raw_u64(seed, stream, start, count, device), 40)
    return (r.to(torch.float32) + 0.5) * (1.0 / 16777216.0)


def normal(seed, stream, start, count, device="cpu"):
    """float32 standard normals (Box-Muller on two 24-bit uniforms of the same counter)."""
    r = raw_u64(seed, stream, start, count, device)
    u1 = (_lsr(r, 40).to(torch.float32) + 0.5) * (1.0 / 16777216.0)
    u2 = ((r & 0xFFFFFF).to(torch.float32) + 0.5) * (1.0 / 16777216.0)
    return torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)


def _choose_channels(seed, stream, plane, head_dim, n):
    """n distinct channel ids of one (layer, head) plane: the n smallest hashes."""
    h = raw_u64(seed, stream, plane * head_dim, head_dim, "cpu")
    return torch.argsort(h, stable=True)[:n]


def make_kv(layers, kv_heads, tokens, head_dim, seed, kind="llama", device="cpu"):
    """fp16 K, V tensors [layers, kv_heads, tokens, head_dim].

    kind "tiny":  N(0,1); 4 key channels per head scaled x20.
    kind "llama": K ~ N(0,1) with ceil(2 % of head_dim) channels per (layer, head) scaled by a
                  factor uniform in [10, 50]; V ~ N(0,1) times a per-token scale log-uniform
                  in [0.5, 4].
    """
    K = torch.empty((layers, kv_heads, tokens, head_dim), dtype=torch.float16, device=device)
    V = torch.empty_like(K)
    per_plane = tokens * head_dim
    if kind == "llama":
        u = uniform01(seed, 5, 0, tokens, device)
        vscale = (0.5 * torch.pow(torch.tensor(8.0, device=device), u)).view(tokens, 1)
    for l in range(layers):
        for h in range(kv_heads):
            plane = l * kv_heads + h
            k = normal(seed, 1, plane * per_plane, per_plane, device).view(tokens, head_dim)
            v = normal(seed, 2, plane * per_plane, per_plane, device).view(tokens, head_dim)
            if kind == "tiny":
                ch = _choose_channels(seed, 3, plane, head_dim, 4).to(device)
                k[:, ch] *= 20.0
            elif kind == "llama":
                n_out = max(1, math.ceil(0.02 * head_dim))
                ch = _choose_channels(seed, 3, plane, head_dim, n_out).to(device)
                f = 10.0 + 40.0 * uniform01(seed, 4, plane * n_out, n_out, device)
                k[:, ch] *= f
                v = v * vscale
            else:
                raise ValueError(kind)
            K[l, h] = k.to(torch.float16)
            V[l, h] = v.to(torch.float16)
    return K, V


def make_scores(tokens, seed, device="cpu"):
    """Per-token scores ~ Uniform(0, 1), float32."""
    return uniform01(seed, 7, 0, tokens, device)


def make_features(tokens, seed, device="cpu"):
    """Controller features [tokens, 6], float32: frequency, quality, attention variance and entropy
    ~ Uniform(0, 1); downstream demand ~ Uniform(0, 1) lifted by 0.5 inside shared segments; segment
    type 0 (private), 0.5 (shared context) or 1 (shared state), constant over segments of 64 tokens."""
    f = torch.stack([uniform01(seed, 20 + i, 0, tokens, device) for i in range(5)], dim=1)
    n_seg = (tokens + 63) // 64
    seg = _lsr(raw_u64(seed, 26, 0, n_seg, device), 62).clamp(max=2)        # 0, 1, 2 (2 twice as likely)
    seg = seg.repeat_interleave(64)[:tokens].to(torch.float32) * 0.5
    f[:, 4] = f[:, 4] + 0.5 * (seg > 0).to(torch.float32)
    return torch.cat([f, seg.view(tokens, 1)], dim=1).contiguous()


def make_controller(seed, device="cpu"):
    """Random-initialised controller weights (trained ones are not available): w1 [64, 6] ~ N(0, 1/6),
    b1 [64] ~ N(0, 0.01), w2 [64] = |N(0, 1/64)| (non-negative, so that scores are non-negative)."""
    w1 = (normal(seed, 30, 0, 64 * 6, device) * (1.0 / math.sqrt(6.0))).view(64, 6).contiguous()
    b1 = normal(seed, 31, 0, 64, device) * 0.1
    w2 = (normal(seed, 32, 0, 64, device) * 0.125).abs()
    return w1, b1, w2


def make_bits_uniform_choice(tokens, seed, device="cpu"):
    """Each token's width drawn uniformly from {2, 4, 8, 16}: a caller-made vector."""
    r = _lsr(raw_u64(seed, 8, 0, tokens, device), 62)
    table = torch.tensor([2, 4, 8, 16], dtype=torch.uint8, device=device)
    return table[r]


def make_bits_constant(tokens, width, device="cpu"):
    return torch.full((tokens,), width, dtype=torch.uint8, device=device)


# The benchmark configurations: shape, value recipe, how the widths are obtained.
CONFIGS = {
    "tiny": dict(layers=1, kv_heads=2, tokens=256, head_dim=128, group_size=32, kind="tiny",
                 data_seed=1001, bits=("choice", 1002)),
    "llama8b_1k_b5": dict(layers=32, kv_heads=8, tokens=1024, head_dim=128, group_size=32, kind="llama",
                          data_seed=2001, bits=("budget", 2002, 5.0)),
    "llama8b_1k_b4": dict(layers=32, kv_heads=8, tokens=1024, head_dim=128, group_size=32, kind="llama",
                          data_seed=2001, bits=("budget", 2002, 4.0)),
    "llama8b_8k_b3": dict(layers=32, kv_heads=8, tokens=8192, head_dim=128, group_size=32, kind="llama",
                          data_seed=3001, bits=("budget", 3002, 3.0)),
    "llama8b_8k_u4_g64": dict(layers=32, kv_heads=8, tokens=8192, head_dim=128, group_size=64, kind="llama",
                              data_seed=4001, bits=("constant", 4)),
    "llama8b_8k_u2_g64": dict(layers=32, kv_heads=8, tokens=8192, head_dim=128, group_size=64, kind="llama",
                              data_seed=4001, bits=("constant", 2)),
    "llama8b_8k_u4_g32_kc": dict(layers=32, kv_heads=8, tokens=8192, head_dim=128, group_size=32, kind="llama",
                                 data_seed=4001, bits=("constant", 4), keys_per_channel=True),
    "llama8b_32k_hops": dict(layers=32, kv_heads=8, tokens=32768, head_dim=128, group_size=32, kind="llama",
                             data_seed=5001, bits=("hops", (5003, 5004, 5005, 5006), (6.0, 4.0, 3.0, 2.0))),
}
