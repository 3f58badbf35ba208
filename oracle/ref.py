"""ctypes front end of the CPU oracle (oracle/qkv_ref.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the benchmark's
CPU-baseline leg.  The product package never imports this module.

All arrays are numpy, host memory.  fp16 tensors are passed as uint16 bit patterns or
float16 arrays (viewed as uint16).
"""
import ctypes
import os

import numpy as np

from . import build as _build

WIDTHS = (2, 4, 8, 16)


class RefDesc(ctypes.Structure):
    _fields_ = [
        ("layers", ctypes.c_int32),
        ("kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("group_size", ctypes.c_int32),
        ("tokens", ctypes.c_int64),
        ("model_id", ctypes.c_uint64),
        ("sender_id", ctypes.c_uint64),
        ("position_offset", ctypes.c_int64),
    ]


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = ctypes.CDLL(path)
        _lib.qkv_ref_half_to_float.restype = ctypes.c_float
        _lib.qkv_ref_half_to_float.argtypes = [ctypes.c_uint16]
        _lib.qkv_ref_float_to_half.restype = ctypes.c_uint16
        _lib.qkv_ref_float_to_half.argtypes = [ctypes.c_float]
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code, where):
        super().__init__(f"oracle {where} returned {code}")
        self.code = code


def _check(rc, where):
    if rc != 0:
        raise OracleError(rc, where)


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def make_desc(layers, kv_heads, tokens, head_dim, group_size, model_id=0, sender_id=0, position_offset=0):
    return RefDesc(layers, kv_heads, head_dim, group_size, tokens, model_id, sender_id, position_offset)


def _counts_arr(counts):
    a = np.ascontiguousarray(np.asarray(counts, dtype=np.int64))
    assert a.shape == (4,)
    return a


def _as_u16(x):
    x = np.ascontiguousarray(x)
    if x.dtype == np.float16:
        return x.view(np.uint16)
    assert x.dtype == np.uint16
    return x


def half_to_float(h):
    return lib().qkv_ref_half_to_float(int(h))


def float_to_half(f):
    return lib().qkv_ref_float_to_half(float(f))


def card_bytes(desc, counts):
    out = ctypes.c_uint64(0)
    c = _counts_arr(counts)
    _check(lib().qkv_ref_card_bytes(ctypes.byref(desc), _ptr(c), ctypes.byref(out)), "card_bytes")
    return out.value


def card_offsets(desc, counts):
    out = np.zeros(11, dtype=np.uint64)
    c = _counts_arr(counts)
    _check(lib().qkv_ref_card_offsets(ctypes.byref(desc), _ptr(c), _ptr(out)), "card_offsets")
    names = ["bits", "slot", "order", "codes2", "meta2", "codes4", "meta4", "codes8", "meta8", "fp16", "total"]
    return {n: int(v) for n, v in zip(names, out)}


def budget_counts(tokens, budget):
    out = np.zeros(4, dtype=np.int64)
    _check(lib().qkv_ref_budget_counts(ctypes.c_int64(tokens), ctypes.c_double(budget), _ptr(out)), "budget_counts")
    return out


def assign_bits(scores, budget):
    scores = np.ascontiguousarray(scores, dtype=np.float32)
    T = scores.shape[0]
    bits = np.zeros(T, dtype=np.uint8)
    counts = np.zeros(4, dtype=np.int64)
    _check(lib().qkv_ref_assign_bits(_ptr(scores), ctypes.c_int64(T), ctypes.c_double(budget), _ptr(bits), _ptr(counts)),
           "assign_bits")
    return bits, counts


def controller_scores(features, w1, b1, w2):
    """Scores of the 6 -> 64 -> 1 controller network; features [T, 6], w1 [64, 6], b1 [64], w2 [64], all float32."""
    features = np.ascontiguousarray(features, dtype=np.float32)
    w1 = np.ascontiguousarray(w1, dtype=np.float32)
    b1 = np.ascontiguousarray(b1, dtype=np.float32)
    w2 = np.ascontiguousarray(w2, dtype=np.float32)
    assert features.ndim == 2 and features.shape[1] == 6 and w1.shape == (64, 6) and b1.shape == (64,) and w2.shape == (64,)
    T = features.shape[0]
    scores = np.zeros(T, dtype=np.float32)
    _check(lib().qkv_ref_controller_scores(_ptr(features), ctypes.c_int64(T), _ptr(w1), _ptr(b1), _ptr(w2), _ptr(scores)),
           "controller_scores")
    return scores


def assign_bits_greedy(scores, budget):
    """Objective-greedy allocator: widths and class counts."""
    scores = np.ascontiguousarray(scores, dtype=np.float32)
    T = scores.shape[0]
    bits = np.zeros(T, dtype=np.uint8)
    counts = np.zeros(4, dtype=np.int64)
    _check(lib().qkv_ref_assign_bits_greedy(_ptr(scores), ctypes.c_int64(T), ctypes.c_double(budget), _ptr(bits),
                                            _ptr(counts)), "assign_bits_greedy")
    return bits, counts


def count_bits(bits):
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    counts = np.zeros(4, dtype=np.int64)
    _check(lib().qkv_ref_count_bits(_ptr(bits), ctypes.c_int64(bits.shape[0]), _ptr(counts)), "count_bits")
    return counts


def compact(bits):
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    T = bits.shape[0]
    slot = np.zeros(T, dtype=np.uint32)
    order = np.zeros(T, dtype=np.uint32)
    counts = np.zeros(4, dtype=np.int64)
    _check(lib().qkv_ref_compact(_ptr(bits), ctypes.c_int64(T), _ptr(slot), _ptr(order), _ptr(counts)), "compact")
    return slot, order, counts


def quantize_group(x, width):
    x = _as_u16(x)
    n = x.shape[0]
    scale = ctypes.c_uint16(0)
    zero = ctypes.c_uint16(0)
    codes = np.zeros(n, dtype=np.uint8)
    _check(lib().qkv_ref_quantize_group(_ptr(x), ctypes.c_int(n), ctypes.c_int(width), ctypes.byref(scale),
                                        ctypes.byref(zero), _ptr(codes)), "quantize_group")
    return scale.value, zero.value, codes


def dequantize_group(codes, scale_h, zero_h):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    out = np.zeros(codes.shape[0], dtype=np.uint16)
    _check(lib().qkv_ref_dequantize_group(_ptr(codes), ctypes.c_int(codes.shape[0]), ctypes.c_uint16(scale_h),
                                          ctypes.c_uint16(zero_h), _ptr(out)), "dequantize_group")
    return out


def pack_codes(codes, width):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    n = codes.shape[0]
    out = np.zeros(n * width // 8, dtype=np.uint8)
    _check(lib().qkv_ref_pack_codes(_ptr(codes), ctypes.c_int(n), ctypes.c_int(width), _ptr(out)), "pack_codes")
    return out


def unpack_codes(packed, n, width):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    out = np.zeros(n, dtype=np.uint8)
    _check(lib().qkv_ref_unpack_codes(_ptr(packed), ctypes.c_int(n), ctypes.c_int(width), _ptr(out)), "unpack_codes")
    return out


def quantize_pack(desc, k, v, bits, counts, capacity=None):
    """Returns the card as a uint8 array of exactly card_bytes (or `capacity`) bytes."""
    k = _as_u16(k)
    v = _as_u16(v)
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    c = _counts_arr(counts)
    n = 2 * desc.layers * desc.kv_heads * desc.tokens * desc.head_dim
    assert k.size * 2 == n and v.size * 2 == n and bits.shape[0] == desc.tokens
    if capacity is None:
        capacity = card_bytes(desc, counts)
    card = np.zeros(capacity, dtype=np.uint8)
    _check(lib().qkv_ref_quantize_pack(ctypes.byref(desc), _ptr(k), _ptr(v), _ptr(bits), _ptr(c), _ptr(card),
                                       ctypes.c_uint64(capacity)), "quantize_pack")
    return card


def quantize_pack_kc(desc, k, v, bits, counts, capacity=None):
    """Uniform card with keys grouped per channel (values per token); same arguments as quantize_pack."""
    k = _as_u16(k)
    v = _as_u16(v)
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    c = _counts_arr(counts)
    if capacity is None:
        capacity = card_bytes(desc, counts)
    card = np.zeros(capacity, dtype=np.uint8)
    _check(lib().qkv_ref_quantize_pack_kc(ctypes.byref(desc), _ptr(k), _ptr(v), _ptr(bits), _ptr(c), _ptr(card),
                                          ctypes.c_uint64(capacity)), "quantize_pack_kc")
    return card


def unpack_dequant_kc(card, expect):
    """Returns (k, v) as uint16 arrays shaped [L, H, T, D] from a card with keys grouped per channel."""
    card = np.ascontiguousarray(card, dtype=np.uint8)
    shape = (expect.layers, expect.kv_heads, expect.tokens, expect.head_dim)
    k = np.zeros(shape, dtype=np.uint16)
    v = np.zeros(shape, dtype=np.uint16)
    _check(lib().qkv_ref_unpack_dequant_kc(_ptr(card), ctypes.c_uint64(card.size), ctypes.byref(expect), _ptr(k), _ptr(v)),
           "unpack_dequant_kc")
    return k, v


def card_peek(card):
    card = np.ascontiguousarray(card, dtype=np.uint8)
    d = RefDesc()
    counts = np.zeros(4, dtype=np.int64)
    avg = ctypes.c_float(0)
    status = ctypes.c_uint32(0)
    _check(lib().qkv_ref_card_peek(_ptr(card), ctypes.c_uint64(card.shape[0]), ctypes.byref(d), _ptr(counts),
                                   ctypes.byref(avg), ctypes.byref(status)), "card_peek")
    return d, counts, avg.value, status.value


def unpack_dequant(card, expect):
    """Returns (k, v) as uint16 arrays shaped [L, H, T, D]."""
    card = np.ascontiguousarray(card, dtype=np.uint8)
    shape = (expect.layers, expect.kv_heads, expect.tokens, expect.head_dim)
    k = np.zeros(shape, dtype=np.uint16)
    v = np.zeros(shape, dtype=np.uint16)
    _check(lib().qkv_ref_unpack_dequant(_ptr(card), ctypes.c_uint64(card.shape[0]), ctypes.byref(expect), _ptr(k),
                                        _ptr(v)), "unpack_dequant")
    return k, v
