"""Pins of the injection oracle's position realignment against the textbook rotary embedding, closed
forms and invariants; no GPU."""
import math

import numpy as np
import pytest

import qkv_synth
from oracle import inject_ref, ref


def f16(a):
    return np.asarray(a, dtype=np.float16)


def rotate(x_f16, D, base, delta):
    return inject_ref.rope_rotate(f16(x_f16).view(np.uint16), *inject_ref.rope_table(D, base, delta)).view(np.float16)


def textbook_rope(x, pos, base):
    """The standard half-split rotary embedding in float64: x [..., D] at position pos."""
    D = x.shape[-1]
    i = np.arange(D // 2, dtype=np.float64)
    ang = pos * base ** (-2.0 * i / D)
    cos = np.concatenate([np.cos(ang), np.cos(ang)])
    sin = np.concatenate([np.sin(ang), np.sin(ang)])
    rot = np.concatenate([-x[..., D // 2:], x[..., :D // 2]], axis=-1)         # rotate_half
    return x * cos + rot * sin


def test_unit_vector_gives_cos_and_sin_of_one_radian():
    # element 0 has frequency base^0 = 1: a shift by one position turns (1, 0) into (cos 1, sin 1).
    # cos 1 = 0.540302 -> 1107 * 2^-11 -> 0x3853;  sin 1 = 0.841471 -> 1723 * 2^-11 -> 0x3ABB
    x = np.zeros((1, 128), np.float16)
    x[0, 0] = 1
    out = rotate(x, 128, 10000.0, 1).view(np.uint16)
    assert out[0, 0] == 0x3853 and out[0, 64] == 0x3ABB
    assert np.count_nonzero(out) == 2
    # the partner element alone turns into (-sin 1, cos 1)
    x[:] = 0
    x[0, 64] = 1
    out = rotate(x, 128, 10000.0, 1).view(np.uint16)
    assert out[0, 0] == 0x3ABB | 0x8000 and out[0, 64] == 0x3853


def test_table_closed_forms():
    c, s = inject_ref.rope_table(128, 10000.0, 0)
    assert np.all(c == 1) and np.all(s == 0)
    c, s = inject_ref.rope_table(128, 10000.0, 7)
    assert c[0] == np.float32(math.cos(7.0)) and s[0] == np.float32(math.sin(7.0))
    # i = 32 of 64: frequency 10000^-0.5 = 0.01
    assert abs(float(c[32]) - math.cos(0.07)) < 1e-7 and abs(float(s[32]) - math.sin(0.07)) < 1e-7
    # frequencies fall geometrically: ratio of consecutive angles is 10000^(-1/64)
    _, s1 = inject_ref.rope_table(128, 10000.0, 1)
    small = np.arcsin(s1[40:].astype(np.float64))
    assert np.allclose(small[1:] / small[:-1], 10000.0 ** (-1 / 64), rtol=1e-5)
    c2, s2 = inject_ref.rope_table(128, 10000.0, -7)
    assert np.array_equal(c2, c) and np.array_equal(s2, -s)
    with pytest.raises(ref.OracleError):
        inject_ref.rope_table(128, 0.0, 1)


@pytest.mark.parametrize("D,base,delta", [(128, 10000.0, 5), (128, 500000.0, 1234), (64, 10000.0, -77), (256, 1e6, 40000)])
def test_matches_textbook_rotary_embedding(D, base, delta):
    # a key cached at position m, realigned by delta, is the key of position m + delta
    rng = np.random.default_rng(D + abs(delta))
    raw = rng.standard_normal((50, D))
    m = 321
    cached = f16(textbook_rope(raw, m, base))
    got = rotate(cached, D, base, delta).astype(np.float64)
    want = textbook_rope(cached.astype(np.float64), delta, base)        # rotations compose
    assert np.max(np.abs(got - want)) <= 2.0 ** -11 * np.max(np.abs(want)) + 1e-6
    direct = textbook_rope(raw, m + delta, base)
    assert np.max(np.abs(got - direct)) < 4e-3 * np.max(np.abs(direct))


def test_scores_depend_on_relative_position_only():
    rng = np.random.default_rng(3)
    D, base = 128, 10000.0
    q, k = rng.standard_normal((2, 20, D))
    qm = f16(textbook_rope(q, 900, base)).astype(np.float64)
    kn = f16(textbook_rope(k, 100, base))
    before = np.sum(qm * kn.astype(np.float64), axis=-1)
    q2 = textbook_rope(q, 900 + 555, base)
    k2 = rotate(kn, D, base, 555).astype(np.float64)
    after = np.sum(q2 * k2, axis=-1)
    assert np.max(np.abs(before - after)) < 0.05


def test_zero_shift_is_the_identity_and_norms_are_kept():
    K, _ = qkv_synth.make_kv(1, 2, 64, 128, 9, "llama")
    x = K.numpy().reshape(-1, 128)
    assert np.array_equal(rotate(x, 128, 10000.0, 0), x)                 # value equality (signs of zeros aside)
    y = rotate(x, 128, 10000.0, 4097).astype(np.float64)
    x64 = x.astype(np.float64)
    n0 = x64[:, :64] ** 2 + x64[:, 64:] ** 2
    n1 = y[:, :64] ** 2 + y[:, 64:] ** 2
    assert np.max(np.abs(n1 - n0) / (n0 + 1e-3)) < 3e-3
    back = rotate(y.astype(np.float16), 128, 10000.0, -4097).astype(np.float64)
    assert np.max(np.abs(back - x64)) <= 3 * 2.0 ** -11 * np.max(np.abs(x64), axis=None)


def test_rounding_steps_are_product_then_fused_then_half():
    # a = b = 2^15 (1 + 2^-10) = 32800 (fp16), table c = s = 1 + 2^-23 (fp32).
    # b*s = 2^15 (1 + 2^-10 + 2^-23 + 2^-33) rounds to fp32 2^15 (1 + 2^-10 + 2^-23): the 2^-18 is lost.
    # a*c is the same product, but inside the fma it stays exact, so x'[0] = a*c - fl32(b*s) = 2^-18 exactly,
    # the fp16 subnormal 64 * 2^-24 = 0x0040.  Two separately rounded products, or both kept exact, give 0.
    # x'[1] = a*c + fl32(a*s) = 65600.0... is past the largest fp16 (ties at 65520) -> +inf.
    x = np.zeros((1, 2), np.float16)
    x[0, 0] = x[0, 1] = 32800
    c = np.array([1 + 2.0 ** -23], np.float32)
    out = inject_ref.rope_rotate(x.view(np.uint16), c, c)
    assert out[0, 0] == 0x0040 and out[0, 1] == 0x7C00
    # the last step rounds the fp32 result to fp16, ties to even: 1 + 2^-11 lies half-way between 0x3C00 and
    # 0x3C01 and goes to the even one, 1 + 3 * 2^-11 half-way between 0x3C01 and 0x3C02 goes up
    x[0, 0], x[0, 1] = 1, 0
    out = inject_ref.rope_rotate(x.view(np.uint16), np.array([1 + 2.0 ** -11], np.float32), np.array([0], np.float32))
    assert out[0, 0] == 0x3C00
    out = inject_ref.rope_rotate(x.view(np.uint16), np.array([1 + 3 * 2.0 ** -11], np.float32), np.array([0], np.float32))
    assert out[0, 0] == 0x3C02


def test_inject_layers_places_rows_and_rotates_keys_only():
    L, H, T, D, G = 3, 2, 40, 128, 32
    K, V = qkv_synth.make_kv(L, H, T, D, 31, "llama")
    bits = qkv_synth.make_bits_uniform_choice(T, 32).numpy()
    counts = ref.count_bits(bits)
    desc = ref.make_desc(L, H, T, D, G)
    card = ref.quantize_pack(desc, K.numpy().view(np.uint16), V.numpy().view(np.uint16), bits, counts)
    dk, dv = ref.unpack_dequant(card, desc)
    cap, prefix = 100, 17
    kl = [np.full((H, cap, D), 0x7E00, np.uint16) for _ in range(2)]
    vl = [np.full((H, cap, D), 0x7E00, np.uint16) for _ in range(2)]
    inject_ref.inject_layers(card, desc, kl, vl, 1, prefix, rope=(10000.0, 9))
    for i in range(2):
        assert np.all(kl[i][:, :prefix] == 0x7E00) and np.all(kl[i][:, prefix + T:] == 0x7E00)
        assert np.array_equal(vl[i][:, prefix:prefix + T], dv[1 + i])
        want = rotate(dk[1 + i].view(np.float16), D, 10000.0, 9).view(np.uint16)
        assert np.array_equal(kl[i][:, prefix:prefix + T], want)
        assert not np.array_equal(kl[i][:, prefix:prefix + T], dk[1 + i])
    kl2 = [np.zeros((H, cap, D), np.uint16)]
    vl2 = [np.zeros((H, cap, D), np.uint16)]
    inject_ref.inject_layers(card, desc, kl2, vl2, 0, 0)
    assert np.array_equal(kl2[0][:, :T], dk[0]) and np.array_equal(vl2[0][:, :T], dv[0])
