"""CPU oracle for receiver-side injection into per-layer caches (paper Sec. 4.2.2) with optional
position realignment of the keys (Sec. 3.2, challenge 2; Sec. 4.2.1 position-offset field).

TEST INFRASTRUCTURE ONLY: imported by tests/ and the smoke check, never by the product package.

Injection is the dense dequantization (oracle.ref.unpack_dequant) followed by plain indexing: layer l's
keys go to a tensor of shape [kv_heads, capacity, head_dim] at token positions prefix .. prefix+T-1, the
layout of one layer of a per-layer key/value cache for one sequence.  Realignment rotates every
injected key row (oracle/inject_ref.cpp); values are not position dependent and are left alone.
"""
import ctypes

import numpy as np

from . import ref


def rope_table(head_dim, base, delta):
    """(cos, sin) float32 arrays [head_dim / 2] for a shift of `delta` positions."""
    c = np.zeros(head_dim // 2, dtype=np.float32)
    s = np.zeros(head_dim // 2, dtype=np.float32)
    L = ref.lib()
    rc = L.qkv_ref_rope_table(ctypes.c_int32(head_dim), ctypes.c_double(base), ctypes.c_int64(delta), ref._ptr(c), ref._ptr(s))
    if rc:
        raise ref.OracleError(rc, "rope_table")
    return c, s


def rope_rotate(rows_u16, cos_t, sin_t):
    """rows_u16: uint16 array [..., head_dim] of fp16 bit patterns; returns the rotated copy."""
    out = np.ascontiguousarray(rows_u16, dtype=np.uint16).copy()
    D = out.shape[-1]
    rc = ref.lib().qkv_ref_rope_rotate(ref._ptr(out), ctypes.c_int64(out.size // D), ctypes.c_int32(D),
                                       ref._ptr(np.ascontiguousarray(cos_t, dtype=np.float32)),
                                       ref._ptr(np.ascontiguousarray(sin_t, dtype=np.float32)))
    if rc:
        raise ref.OracleError(rc, "rope_rotate")
    return out


def inject_layers(card, desc, k_layers, v_layers, layer_begin, prefix, rope=None, keys_per_channel=False):
    """Writes layers layer_begin .. layer_begin + len(k_layers) - 1 of the card into the given per-layer
    uint16 arrays [kv_heads, capacity, head_dim] at token positions prefix .. prefix + T - 1.
    rope: None or (base, delta).  keys_per_channel: the card is a uniform card with per-channel key groups."""
    K, V = (ref.unpack_dequant_kc if keys_per_channel else ref.unpack_dequant)(card, desc)      # [L, H, T, D] uint16
    T, D = desc.tokens, desc.head_dim
    table = rope_table(D, rope[0], rope[1]) if rope is not None else None
    for i, (kl, vl) in enumerate(zip(k_layers, v_layers)):
        k = K[layer_begin + i]
        if table is not None:
            k = rope_rotate(k, *table)
        kl[:, prefix:prefix + T, :] = k
        vl[:, prefix:prefix + T, :] = V[layer_begin + i]
