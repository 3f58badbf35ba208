"""Pins for the attention oracle (oracle/attend_ref.py): closed forms, special cases and an
independent pure-Python evaluation, none of which retypes the oracle's vectorised formula."""
import math

import numpy as np

import qkv_synth
from oracle import attend_ref, ref


def rand_case(L=2, H=2, rep=2, T=37, D=16, seed=0):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((L, H * rep, D)).astype(np.float16)
    K = rng.standard_normal((L, H, T, D)).astype(np.float16)
    V = rng.standard_normal((L, H, T, D)).astype(np.float16)
    return q, K, V


def test_single_token_returns_its_value_row():
    q, K, V = rand_case(T=1)
    o, lse = attend_ref.attend_dense(q, K, V, 0.25)
    for l in range(2):
        for hq in range(4):
            assert np.array_equal(o[l, hq], V[l, hq // 2, 0].astype(np.float64))
            s = 0.25 * float(np.dot(K[l, hq // 2, 0].astype(np.float64), q[l, hq].astype(np.float64)))
            assert abs(lse[l, hq] - s) < 1e-12


def test_zero_query_and_identical_keys_give_the_mean_of_v():
    q, K, V = rand_case(T=50)
    o, lse = attend_ref.attend_dense(np.zeros_like(q), K, V, 0.3)
    assert np.allclose(o, V.astype(np.float64).mean(axis=2).repeat(2, axis=1), rtol=0, atol=1e-13)
    assert np.allclose(lse, math.log(50), atol=1e-13)
    K2 = np.broadcast_to(K[:, :, :1, :], K.shape)
    o2, lse2 = attend_ref.attend_dense(q, K2, V, 0.3)
    assert np.allclose(o2, V.astype(np.float64).mean(axis=2).repeat(2, axis=1), atol=1e-13)


def test_two_tokens_logistic_closed_form():
    q, K, V = rand_case(T=2, seed=3)
    o, lse = attend_ref.attend_dense(q, K, V, 0.5)
    for l in range(2):
        for hq in range(4):
            h = hq // 2
            s0 = 0.5 * sum(float(a) * float(b) for a, b in zip(K[l, h, 0], q[l, hq]))
            s1 = 0.5 * sum(float(a) * float(b) for a, b in zip(K[l, h, 1], q[l, hq]))
            w0 = 1.0 / (1.0 + math.exp(s1 - s0))
            want = w0 * V[l, h, 0].astype(np.float64) + (1 - w0) * V[l, h, 1].astype(np.float64)
            assert np.allclose(o[l, hq], want, atol=1e-13)
            assert abs(lse[l, hq] - (max(s0, s1) + math.log1p(math.exp(-abs(s0 - s1))))) < 1e-12


def test_dominant_key_selects_its_value():
    q, K, V = rand_case(T=20, seed=4)
    K = K.copy()
    K[:, :, 7, :] = 0
    # make token 7's key point along the first query head of each kv head, far ahead of the rest
    for l in range(2):
        for h in range(2):
            K[l, h, 7] = (q[l, 2 * h].astype(np.float32) * 40).astype(np.float16)
    o, _ = attend_ref.attend_dense(q, K, V, 1.0)
    for l in range(2):
        for h in range(2):
            assert np.allclose(o[l, 2 * h], V[l, h, 7].astype(np.float64), atol=1e-6)


def test_token_permutation_and_key_shift_invariance():
    q, K, V = rand_case(T=64, seed=5)
    o, lse = attend_ref.attend_dense(q, K, V, 0.2)
    perm = np.random.default_rng(6).permutation(64)
    o2, lse2 = attend_ref.attend_dense(q, K[:, :, perm], V[:, :, perm], 0.2)
    assert np.allclose(o, o2, atol=1e-13) and np.allclose(lse, lse2, atol=1e-13)
    # adding one vector c to every key shifts all scores of a head by scale*<q, c>: o unchanged, lse shifted
    c = np.random.default_rng(7).standard_normal(16)
    o3, lse3 = attend_ref.attend_dense(q, K.astype(np.float64) + c, V, 0.2)
    shift = 0.2 * (q.astype(np.float64) @ c)
    assert np.allclose(o, o3, atol=1e-12) and np.allclose(lse3, lse + shift, atol=1e-12)


def test_merge_of_two_disjoint_token_sets():
    q, K, V = rand_case(T=90, seed=8)
    o, lse = attend_ref.attend_dense(q, K, V, 0.25)
    oa, la = attend_ref.attend_dense(q, K[:, :, :33], V[:, :, :33], 0.25)
    ob, lb = attend_ref.attend_dense(q, K[:, :, 33:], V[:, :, 33:], 0.25)
    m = np.maximum(la, lb)
    wa, wb = np.exp(la - m), np.exp(lb - m)
    merged = (wa[..., None] * oa + wb[..., None] * ob) / (wa + wb)[..., None]
    assert np.allclose(o, merged, atol=1e-13)
    assert np.allclose(lse, m + np.log(wa + wb), atol=1e-13)


def test_pure_python_loops_on_a_tiny_case():
    q, K, V = rand_case(L=1, H=2, rep=3, T=5, D=4, seed=9)
    o, lse = attend_ref.attend_dense(q, K, V, 0.7)
    for hq in range(6):
        h = hq // 3
        s = [0.7 * sum(float(K[0, h, t, d]) * float(q[0, hq, d]) for d in range(4)) for t in range(5)]
        z = sum(math.exp(x) for x in s)
        for d in range(4):
            want = sum(math.exp(s[t]) * float(V[0, h, t, d]) for t in range(5)) / z
            assert abs(o[0, hq, d] - want) < 1e-13
        assert abs(lse[0, hq] - math.log(z)) < 1e-13


def test_card_attend_uses_the_dequantized_cache():
    # over a card, attention sees exactly what injection would rebuild; raw fp16 tokens are seen unchanged
    L, H, T, D, G = 1, 2, 48, 64, 32
    K, V = qkv_synth.make_kv(L, H, T, D, 77, "llama")
    bits = qkv_synth.make_bits_uniform_choice(T, 78).numpy()
    counts = ref.count_bits(bits)
    d = ref.make_desc(L, H, T, D, G)
    card = ref.quantize_pack(d, K.numpy(), V.numpy(), bits, counts)
    q = np.random.default_rng(1).standard_normal((L, 4, D)).astype(np.float16)
    o, lse = attend_ref.card_attend(card, d, q, D ** -0.5)
    kq, vq = ref.unpack_dequant(card, d)
    o2, lse2 = attend_ref.attend_dense(q, kq.view(np.float16), vq.view(np.float16), D ** -0.5)
    assert np.array_equal(o, o2) and np.array_equal(lse, lse2)
    all16 = np.full(T, 16, dtype=np.uint8)
    card16 = ref.quantize_pack(d, K.numpy(), V.numpy(), all16, ref.count_bits(all16))
    o16, _ = attend_ref.card_attend(card16, d, q, D ** -0.5)
    od, _ = attend_ref.attend_dense(q, K.numpy(), V.numpy(), D ** -0.5)
    assert np.array_equal(o16, od)


def test_card_attend_over_per_channel_key_groups():
    # the grouping of the keys is part of what the card means: the same definition over the cache that a per-channel
    # card dequantizes to; a zero query makes the keys irrelevant (o = mean of the values, which both groupings
    # quantize alike); keys constant along the tokens of a block are exact under per-channel groups, so there the
    # result equals attention over the keys themselves
    L, H, T, D, G = 1, 2, 64, 64, 32
    K, V = qkv_synth.make_kv(L, H, T, D, 79, "llama")
    bits = np.full(T, 4, dtype=np.uint8)
    counts = ref.count_bits(bits)
    d = ref.make_desc(L, H, T, D, G)
    card_kc = ref.quantize_pack_kc(d, K.numpy(), V.numpy(), bits, counts)
    card_pt = ref.quantize_pack(d, K.numpy(), V.numpy(), bits, counts)
    q = np.random.default_rng(2).standard_normal((L, 4, D)).astype(np.float16)
    o, lse = attend_ref.card_attend(card_kc, d, q, D ** -0.5, keys_per_channel=True)
    kq, vq = ref.unpack_dequant_kc(card_kc, d)
    o2, lse2 = attend_ref.attend_dense(q, kq.view(np.float16), vq.view(np.float16), D ** -0.5)
    assert np.array_equal(o, o2) and np.array_equal(lse, lse2)
    o_pt, _ = attend_ref.card_attend(card_pt, d, q, D ** -0.5)
    assert not np.array_equal(o, o_pt)                       # the two groupings round the keys differently
    zero = np.zeros_like(q)
    oz, lz = attend_ref.card_attend(card_kc, d, zero, 1.0, keys_per_channel=True)
    ozp, _ = attend_ref.card_attend(card_pt, d, zero, 1.0)
    assert np.array_equal(oz, ozp) and np.allclose(lz, math.log(T), atol=1e-14)
    Kc = K.numpy().copy()
    Kc[:, :, :32, :] = Kc[:, :, :1, :]                      # every channel constant over each block of 32 tokens
    Kc[:, :, 32:, :] = Kc[:, :, 32:33, :]
    card_c = ref.quantize_pack_kc(d, Kc, V.numpy(), bits, counts)
    oc, lc = attend_ref.card_attend(card_c, d, q, D ** -0.5, keys_per_channel=True)
    _, vqc = ref.unpack_dequant_kc(card_c, d)
    od, ld = attend_ref.attend_dense(q, Kc, vqc.view(np.float16), D ** -0.5)
    assert np.array_equal(oc, od) and np.array_equal(lc, ld)
