"""Pins of the oracle's card variant with keys grouped per channel (uniform cards), against the already
pinned per-token quantizer (by transposition), hand-made cases, and the property that motivates the
scheme; no GPU."""
import numpy as np
import pytest

import qkv_synth
from oracle import ref

WIDTH_CLASS = {2: 0, 4: 1, 8: 2}


def make(L, H, T, D, width, seed, kind="llama"):
    K, V = qkv_synth.make_kv(L, H, T, D, seed, kind)
    bits = np.full(T, width, np.uint8)
    counts = [0, 0, 0, 0]
    counts[WIDTH_CLASS[width]] = T
    return K.numpy().view(np.uint16), V.numpy().view(np.uint16), bits, counts


def transposed_blocks(K, D):
    """K [L, H, T, D] -> K' [L, H, T * D / 64, 64]: row (tb, d / 2) holds tokens 32 tb .. 32 tb + 31 of channel d
    (d even) followed by the same tokens of channel d + 1."""
    L, H, T, _ = K.shape
    blocks = K.reshape(L, H, T // 32, 32, D)                    # [.., tb, i, d]
    cols = blocks.transpose(0, 1, 2, 4, 3)                      # [.., tb, d, i]
    return np.ascontiguousarray(cols.reshape(L, H, (T // 32) * (D // 2), 64))


@pytest.mark.parametrize("width", [2, 4, 8])
@pytest.mark.parametrize("D", [64, 128])
def test_key_sections_equal_the_per_token_card_of_the_transposed_cache(width, D):
    L, H, T = 2, 2, 96
    K, V, bits, counts = make(L, H, T, D, width, 7 + width + D)
    d = ref.make_desc(L, H, T, D, 32)
    card = ref.quantize_pack_kc(d, K, V, bits, counts)
    off = ref.card_offsets(d, counts)
    # the same key values as a per-token problem: one "token" per pair of channels and token block
    Kt = transposed_blocks(K, D)
    T2 = Kt.shape[2]
    d2 = ref.make_desc(L, H, T2, 64, 32)
    counts2 = [0, 0, 0, 0]
    counts2[WIDTH_CLASS[width]] = T2
    card2 = ref.quantize_pack(d2, Kt, Kt, np.full(T2, width, np.uint8), counts2)
    off2 = ref.card_offsets(d2, counts2)
    key_codes = L * H * T * D * width // 8
    key_meta = L * H * T * (D // 32) * 4
    cs, ms = "codes%d" % width, "meta%d" % width
    assert np.array_equal(card[off[cs]:off[cs] + key_codes], card2[off2[cs]:off2[cs] + key_codes])
    assert np.array_equal(card[off[ms]:off[ms] + key_meta], card2[off2[ms]:off2[ms] + key_meta])
    # and the decoded keys are the decoded transposed cache, transposed back
    k1, v1 = ref.unpack_dequant_kc(card, d)
    k2, _ = ref.unpack_dequant(card2, d2)
    assert np.array_equal(transposed_blocks(k1, D), k2)


@pytest.mark.parametrize("width", [2, 4, 8])
def test_everything_but_the_key_sections_is_the_per_token_card(width):
    L, H, T, D = 1, 3, 64, 128
    K, V, bits, counts = make(L, H, T, D, width, 17)
    d = ref.make_desc(L, H, T, D, 32, 5, 6, 7)
    kc = ref.quantize_pack_kc(d, K, V, bits, counts)
    pt = ref.quantize_pack(d, K, V, bits, counts)
    off = ref.card_offsets(d, counts)
    cs, ms = "codes%d" % width, "meta%d" % width
    key_codes = L * H * T * D * width // 8
    key_meta = L * H * T * (D // 32) * 4
    same = np.ones(kc.size, bool)
    same[off[cs]:off[cs] + key_codes] = False
    same[off[ms]:off[ms] + key_meta] = False
    same[188:192] = False                                        # the flags word
    assert np.array_equal(kc[same], pt[same])
    assert kc[188:192].view(np.uint32)[0] == 1 and pt[188:192].view(np.uint32)[0] == 0
    assert not np.array_equal(kc[off[cs]:off[cs] + key_codes], pt[off[cs]:off[cs] + key_codes])
    # values decode the same from both
    _, v_kc = ref.unpack_dequant_kc(kc, d)
    _, v_pt = ref.unpack_dequant(pt, d)
    assert np.array_equal(v_kc, v_pt)


def test_constant_channels_are_exact():
    # every channel constant over the tokens: each key group has range 0, so keys come back exactly,
    # while per-token groups (32 different channels) lose most of it at 2 bits
    L, H, T, D = 1, 1, 64, 64
    K = np.tile(np.linspace(-8, 8, D).astype(np.float16), (L, H, T, 1))
    V = np.zeros_like(K)
    bits = np.full(T, 2, np.uint8)
    d = ref.make_desc(L, H, T, D, 32)
    card = ref.quantize_pack_kc(d, K.view(np.uint16), V.view(np.uint16), bits, [T, 0, 0, 0])
    k, _ = ref.unpack_dequant_kc(card, d)
    assert np.array_equal(k, K.view(np.uint16))
    off = ref.card_offsets(d, [T, 0, 0, 0])
    assert not card[off["codes2"]:off["codes2"] + T * D // 4].any()          # all codes 0
    meta = card[off["meta2"]:off["meta2"] + T * (D // 32) * 4].view(np.uint16).reshape(T // 32, D, 2)
    assert not meta[:, :, 0].any()                                           # all scales 0
    assert np.array_equal(meta[0, :, 1], K.view(np.uint16)[0, 0, 0])         # zero = the channel's value
    pt = ref.quantize_pack(d, K.view(np.uint16), V.view(np.uint16), bits, [T, 0, 0, 0])
    k_pt, _ = ref.unpack_dequant(pt, d)
    assert np.abs(k_pt.view(np.float16).astype(np.float64) - K).max() > 1.0


@pytest.mark.parametrize("width", [2, 4])
def test_per_channel_groups_contain_the_outlier_channels(width):
    # what the scheme is for: a few key channels are 10-50x larger than the rest; grouped per token they
    # stretch every group's range, grouped per channel they only cost their own groups
    L, H, T, D = 2, 2, 256, 128
    K, V, bits, counts = make(L, H, T, D, width, 23)
    d = ref.make_desc(L, H, T, D, 32)
    x = K.view(np.float16).astype(np.float64)
    k_kc, _ = ref.unpack_dequant_kc(ref.quantize_pack_kc(d, K, V, bits, counts), d)
    k_pt, _ = ref.unpack_dequant(ref.quantize_pack(d, K, V, bits, counts), d)
    big = np.abs(x).mean(axis=2, keepdims=True) > 5                   # the outlier channels
    small = np.broadcast_to(~big, x.shape)
    err_kc = ((k_kc.view(np.float16).astype(np.float64) - x)[small] ** 2).mean()
    err_pt = ((k_pt.view(np.float16).astype(np.float64) - x)[small] ** 2).mean()
    assert big.sum() > 0
    assert err_pt > 20 * err_kc


def test_error_stays_within_half_a_step_of_the_group():
    L, H, T, D, width = 1, 2, 96, 128, 4
    K, V, bits, counts = make(L, H, T, D, width, 29)
    d = ref.make_desc(L, H, T, D, 32)
    card = ref.quantize_pack_kc(d, K, V, bits, counts)
    k, _ = ref.unpack_dequant_kc(card, d)
    off = ref.card_offsets(d, counts)
    meta = card[off["meta4"]:off["meta4"] + L * H * T * (D // 32) * 4].view(np.float16).reshape(L, H, T // 32, D, 2)
    scale = meta[..., 0].astype(np.float64)                           # [L, H, tb, d]
    x = K.view(np.float16).astype(np.float64).reshape(L, H, T // 32, 32, D)
    y = k.view(np.float16).astype(np.float64).reshape(L, H, T // 32, 32, D)
    bound = scale[:, :, :, None, :] * 0.5 * (1 + 2.0 ** -9) + 2.0 ** -11 * np.abs(y) + 1e-7
    assert np.all(np.abs(x - y) <= bound)
    # group minimum comes back exactly (code 0 decodes to zero = min)
    assert np.array_equal(y.min(axis=3), x.min(axis=3))


def test_variant_errors_and_mutual_refusal():
    L, H, T, D = 1, 1, 64, 64
    K, V, bits, counts = make(L, H, T, D, 4, 31)
    d = ref.make_desc(L, H, T, D, 32)
    with pytest.raises(ref.OracleError):                                  # tokens not a multiple of 32
        K2, V2, b2, c2 = make(L, H, 48, D, 4, 31)
        ref.quantize_pack_kc(ref.make_desc(L, H, 48, D, 32), K2, V2, b2, c2)
    with pytest.raises(ref.OracleError):                                  # group size 64
        ref.quantize_pack_kc(ref.make_desc(L, H, T, D, 64), K, V, bits, counts)
    with pytest.raises(ref.OracleError):                                  # not uniform
        mixed = bits.copy()
        mixed[:32] = 2
        ref.quantize_pack_kc(d, K, V, mixed, [32, 32, 0, 0])
    with pytest.raises(ref.OracleError):                                  # fp16 rows have no groups to regroup
        ref.quantize_pack_kc(d, K, V, np.full(T, 16, np.uint8), [0, 0, 0, T])
    kc = ref.quantize_pack_kc(d, K, V, bits, counts)
    pt = ref.quantize_pack(d, K, V, bits, counts)
    with pytest.raises(ref.OracleError):
        ref.unpack_dequant(kc, d)
    with pytest.raises(ref.OracleError):
        ref.unpack_dequant_kc(pt, d)
    assert ref.card_peek(kc)[1].tolist() == counts
