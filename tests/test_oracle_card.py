"""Pins for the oracle's card-level logic: geometry, compaction, allocator, full cards.

Checked against closed forms, hand-made fixtures, brute force and structural invariants;
offsets used to look into a card are recomputed here from the layout description.
"""
import os

import numpy as np
import pytest
import torch

import qkv_synth
from oracle import ref

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
WIDTHS = (2, 4, 8, 16)


def golden_rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                yield [part.split() for part in line.split("|")]


def al(x):
    return (x + 255) // 256 * 256


def layout(L, H, T, D, G, counts):
    """Section offsets written out from the layout description (independent of the oracle)."""
    P = 2 * L * H
    off = {}
    o = 256
    off["bits"] = o; o += al(T)
    off["slot"] = o; o += al(4 * T)
    off["order"] = o; o += al(4 * T)
    for c, w in enumerate((2, 4, 8)):
        off["codes%d" % w] = o; o += al(P * counts[c] * D * w // 8)
        off["meta%d" % w] = o; o += al(P * counts[c] * (D // G) * 4)
    off["fp16"] = o; o += al(P * counts[3] * D * 2)
    off["total"] = o
    return off


# ----------------------------------------------------------------------------- geometry


@pytest.mark.parametrize("shape,counts,total", [(r[0], r[1], r[2]) for r in golden_rows("card_sizes.txt")])
def test_card_bytes_golden(shape, counts, total):
    L, H, T, D, G = map(int, shape)
    counts = list(map(int, counts))
    d = ref.make_desc(L, H, T, D, G)
    assert ref.card_bytes(d, counts) == int(total[0])


def test_card_offsets_closed_form_random():
    rng = np.random.default_rng(3)
    for _ in range(200):
        L, H = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        D = int(rng.choice([64, 128, 256]))
        G = int(rng.choice([g for g in (32, 64, 128) if g <= D]))
        T = int(rng.integers(1, 3000))
        cuts = np.sort(rng.integers(0, T + 1, size=3))
        counts = [int(cuts[0]), int(cuts[1] - cuts[0]), int(cuts[2] - cuts[1]), int(T - cuts[2])]
        d = ref.make_desc(L, H, T, D, G)
        assert ref.card_offsets(d, counts) == layout(L, H, T, D, G, counts)
        assert ref.card_bytes(d, counts) == layout(L, H, T, D, G, counts)["total"]


def test_code_bytes_ratio_is_sixteen_over_width():
    # Paper Sec. 3.1: Q4 stores about 0.5 byte per element, a 4x reduction; codes alone give exactly 16/w.
    L, H, T, D, G = 4, 2, 1024, 128, 32
    P = 2 * L * H
    for c, w in enumerate((2, 4, 8)):
        counts = [0, 0, 0, 0]
        counts[c] = T
        off = ref.card_offsets(ref.make_desc(L, H, T, D, G), counts)
        code_bytes = off["meta%d" % w] - off["codes%d" % w]
        assert code_bytes * w == P * T * D * 2 * w * w // 16  # i.e. fp16 bytes / code bytes == 16 / w
        assert (P * T * D * 2) / code_bytes == 16 / w


def test_card_bytes_errors():
    d = ref.make_desc(1, 1, 16, 128, 32)
    with pytest.raises(ref.OracleError):
        ref.card_bytes(d, [1, 1, 1, 1])           # counts do not sum to T
    with pytest.raises(ref.OracleError):
        ref.card_bytes(d, [-1, 17, 0, 0])
    with pytest.raises(ref.OracleError):
        ref.card_bytes(ref.make_desc(1, 1, 16, 128, 48), [16, 0, 0, 0])  # G does not divide D
    with pytest.raises(ref.OracleError):
        ref.card_bytes(ref.make_desc(0, 1, 16, 128, 32), [16, 0, 0, 0])


# ----------------------------------------------------------------------------- compaction


def test_compact_brute_force_and_permutation_properties():
    rng = np.random.default_rng(9)
    for T in [1, 2, 7, 64, 257, 1000]:
        bits = rng.choice(np.array([2, 4, 8, 16], dtype=np.uint8), size=T)
        slot, order, counts = ref.compact(bits)
        # brute force O(T^2)
        for t in range(T):
            assert slot[t] == sum(1 for u in range(t) if bits[u] == bits[t])
        assert counts.tolist() == [int((bits == w).sum()) for w in WIDTHS]
        assert sorted(order.tolist()) == list(range(T))
        base = np.concatenate([[0], np.cumsum(counts)[:-1]])
        for c, w in enumerate(WIDTHS):
            seg = order[base[c]:base[c] + counts[c]]
            assert np.all(bits[seg] == w)
            assert np.all(np.diff(seg.astype(np.int64)) > 0)
            assert np.array_equal(slot[seg], np.arange(counts[c], dtype=np.uint32))


def test_compact_rejects_other_widths():
    with pytest.raises(ref.OracleError):
        ref.compact(np.array([2, 4, 3, 16], dtype=np.uint8))


# ----------------------------------------------------------------------------- allocator


@pytest.mark.parametrize("T,budget,counts", [(int(r[0][0]), float(r[1][0]), list(map(int, r[2]))) for r in golden_rows("budget_counts.txt")])
def test_budget_counts_golden(T, budget, counts):
    assert ref.budget_counts(T, budget).tolist() == counts


def test_budget_counts_never_exceed_budget():
    rng = np.random.default_rng(4)
    for _ in range(2000):
        T = int(rng.integers(1, 100000))
        bm = int(rng.integers(2000, 16001))
        c = ref.budget_counts(T, bm / 1000.0)
        assert c.min() >= 0 and c.sum() == T
        assert (2 * c[0] + 4 * c[1] + 8 * c[2] + 16 * c[3]) * 1000 <= bm * T   # sum b(t) <= budget * T (paper Sec. 3.3)
    for bad in [1.99, 16.01, float("nan"), float("inf"), -3.0]:
        with pytest.raises(ref.OracleError):
            ref.budget_counts(100, bad)


def test_assign_bits_rank_rule_and_ties():
    rng = np.random.default_rng(12)
    T = 1000
    scores = rng.random(T).astype(np.float32)
    bits, counts = ref.assign_bits(scores, 5.0)
    assert counts.tolist() == [300, 400, 250, 50]
    assert ref.count_bits(bits).tolist() == counts.tolist()
    # monotone: a higher score never gets fewer bits (scores distinct here)
    o = np.argsort(-scores, kind="stable")
    assert np.all(np.diff(bits[o].astype(int)) <= 0)
    # permutation equivariance for distinct scores
    perm = rng.permutation(T)
    bits_p, _ = ref.assign_bits(scores[perm], 5.0)
    assert np.array_equal(bits_p, bits[perm])
    # ties: the lower index wins
    s = np.zeros(10, dtype=np.float32)
    b, c = ref.assign_bits(s, 9.0)
    want = []
    for w, n in zip((16, 8, 4, 2), c[::-1]):
        want += [w] * int(n)
    assert b.tolist() == want
    # -0 ranks below +0
    s = np.array([-0.0, 0.0, -0.0, 0.0], dtype=np.float32)
    b, c = ref.assign_bits(s, 9.0)
    hi = [i for i in np.argsort(-b.astype(int), kind="stable")[:2]]
    assert sorted(hi) == [1, 3]
    # ends of the budget range
    assert set(ref.assign_bits(scores, 2.0)[0].tolist()) == {2}
    assert set(ref.assign_bits(scores, 16.0)[0].tolist()) == {16}


def test_assign_bits_matches_sort_by_negated_score():
    # independent formulation: numpy lexsort on (index, -score)
    rng = np.random.default_rng(13)
    T = 4096
    scores = np.round(rng.random(T) * 50).astype(np.float32) / 50   # many ties
    for budget in [2.5, 3.0, 4.0, 6.0, 11.0]:
        bits, counts = ref.assign_bits(scores, budget)
        rank = np.lexsort((np.arange(T), -scores.astype(np.float64)))
        want = np.empty(T, dtype=np.uint8)
        n2, n4, n8, n16 = counts.tolist()
        want[rank[:n16]] = 16
        want[rank[n16:n16 + n8]] = 8
        want[rank[n16 + n8:n16 + n8 + n4]] = 4
        want[rank[n16 + n8 + n4:]] = 2
        assert np.array_equal(bits, want)


# ----------------------------------------------------------------------------- whole cards


def tiny_problem(L=1, H=2, T=96, D=128, G=32, seed=1001, kind="tiny", bits_seed=1002):
    K, V = qkv_synth.make_kv(L, H, T, D, seed, kind)
    bits = qkv_synth.make_bits_uniform_choice(T, bits_seed).numpy()
    d = ref.make_desc(L, H, T, D, G, model_id=0x1122334455667788, sender_id=42, position_offset=-7)
    return d, K.numpy(), V.numpy(), bits


def test_header_fields_at_documented_offsets():
    d, K, V, bits = tiny_problem()
    counts = ref.count_bits(bits)
    card = ref.quantize_pack(d, K, V, bits, counts)
    fields = {r[0][2]: (int(r[0][0]), int(r[0][1])) for r in golden_rows("header_fields.txt")}
    assert sum(sz for _, sz in fields.values()) == 256

    def u(name, idx=0, width=None):
        o, sz = fields[name]
        width = width or sz
        return int.from_bytes(card[o + idx * width:o + (idx + 1) * width].tobytes(), "little")

    assert card[:8].tobytes() == b"QKVCARD\0"
    assert u("version") == 1 and u("header_bytes") == 256
    assert (u("layers"), u("kv_heads"), u("head_dim"), u("group_size"), u("tokens")) == (1, 2, 128, 32, 96)
    assert [u("count", i, 8) for i in range(4)] == counts.tolist()
    off = layout(1, 2, 96, 128, 32, counts.tolist())
    assert u("total_bytes") == off["total"] == card.shape[0]
    assert (u("off_bits"), u("off_slot"), u("off_order")) == (off["bits"], off["slot"], off["order"])
    assert [u("off_codes", i, 8) for i in range(3)] == [off["codes2"], off["codes4"], off["codes8"]]
    assert [u("off_meta", i, 8) for i in range(3)] == [off["meta2"], off["meta4"], off["meta8"]]
    assert u("off_fp16") == off["fp16"]
    assert u("model_id") == 0x1122334455667788 and u("sender_id") == 42
    assert u("position_offset") == (-7) % (1 << 64)
    avg = np.frombuffer(card[184:188].tobytes(), dtype=np.float32)[0]
    assert avg == np.float32(float(bits.astype(np.int64).sum()) / 96)   # achieved average bits (paper Sec. 4.2.1)
    assert u("flags") == 0 and u("status") == 0
    assert not card[196:256].any()


def test_card_rows_sit_where_the_layout_says_and_pads_are_zero():
    L, H, T, D, G = 2, 2, 77, 128, 32
    d, K, V, bits = tiny_problem(L, H, T, D, G, seed=7, bits_seed=8)
    counts = ref.count_bits(bits).tolist()
    card = ref.quantize_pack(d, K, V, bits, counts)
    off = layout(L, H, T, D, G, counts)
    slot, order, _ = ref.compact(bits)
    assert np.array_equal(card[off["bits"]:off["bits"] + T], bits)
    assert np.array_equal(card[off["slot"]:off["slot"] + 4 * T].view(np.uint32), slot)
    assert np.array_equal(card[off["order"]:off["order"] + 4 * T].view(np.uint32), order)
    planes = np.concatenate([K.reshape(L * H, T, D), V.reshape(L * H, T, D)]).view(np.uint16)
    P = 2 * L * H
    used = np.zeros(card.shape[0], dtype=bool)
    used[:256] = True
    used[off["bits"]:off["bits"] + T] = True
    used[off["slot"]:off["slot"] + 4 * T] = True
    used[off["order"]:off["order"] + 4 * T] = True
    for p in range(P):
        for t in range(T):
            w = int(bits[t]); c = WIDTHS.index(w); j = int(slot[t]); n = counts[c]
            row = planes[p, t]
            if w == 16:
                o = off["fp16"] + (p * n + j) * D * 2
                assert np.array_equal(card[o:o + 2 * D].view(np.uint16), row)
                used[o:o + 2 * D] = True
                continue
            R = D * w // 8
            o = off["codes%d" % w] + (p * n + j) * R
            m = off["meta%d" % w] + (p * n + j) * (D // G) * 4
            used[o:o + R] = True
            used[m:m + (D // G) * 4] = True
            for g in range(D // G):
                sh, zh, q = ref.quantize_group(row[g * G:(g + 1) * G], w)
                assert card[m + 4 * g:m + 4 * g + 4].view(np.uint16).tolist() == [sh, zh]
                assert np.array_equal(card[o + g * G * w // 8:o + (g + 1) * G * w // 8], ref.pack_codes(q, w))
    assert not card[~used].any()      # every byte outside a documented field is zero padding


def test_all_fp16_card_is_a_bitwise_passthrough():
    L, H, T, D, G = 1, 2, 40, 128, 32
    rng = np.random.default_rng(1)
    K = rng.integers(0, 65536, size=(L, H, T, D), dtype=np.uint64).astype(np.uint16)   # NaN payloads, inf, -0, subnormals
    V = rng.integers(0, 65536, size=(L, H, T, D), dtype=np.uint64).astype(np.uint16)
    K[0, 0, 0, :6] = [0x7C01, 0xFE00, 0x7C00, 0xFC00, 0x8000, 0x0001]
    bits = np.full(T, 16, dtype=np.uint8)
    d = ref.make_desc(L, H, T, D, G)
    card = ref.quantize_pack(d, K, V, bits, [0, 0, 0, T])
    k2, v2 = ref.unpack_dequant(card, d)
    assert np.array_equal(k2, K) and np.array_equal(v2, V)


def test_round_trip_structure_and_error_bound():
    L, H, T, D, G = 2, 2, 200, 128, 32
    d, K, V, bits = tiny_problem(L, H, T, D, G, seed=21, kind="llama", bits_seed=22)
    counts = ref.count_bits(bits)
    card = ref.quantize_pack(d, K, V, bits, counts)
    k2, v2 = ref.unpack_dequant(card, d)
    x = np.concatenate([K.reshape(-1, T, D), V.reshape(-1, T, D)]).astype(np.float64)
    y = np.concatenate([k2.reshape(-1, T, D), v2.reshape(-1, T, D)]).view(np.float16).astype(np.float64)
    # fp16 tokens come back bit-for-bit
    t16 = bits == 16
    assert np.array_equal(K.view(np.uint16)[:, :, t16], k2[:, :, t16])
    assert np.array_equal(V.view(np.uint16)[:, :, t16], v2[:, :, t16])
    # quantized tokens: error <= (max-min)/(2 qmax) per group, with fp16 rounding slack
    for w in (2, 4, 8):
        tw = bits == w
        xg = x[:, tw].reshape(x.shape[0], -1, D // G, G)
        yg = y[:, tw].reshape(xg.shape)
        step = (xg.max(-1) - xg.min(-1)) / ((1 << w) - 1)
        err = np.abs(xg - yg).max(-1)
        assert np.all(err <= step / 2 * (1 + 2.0 ** -9) + 2.0 ** -10 * np.abs(yg).max(-1) + 1e-7)
    # a second hop with the same widths leaves fp16 tokens untouched again
    card2 = ref.quantize_pack(d, k2, v2, bits, counts)
    k3, v3 = ref.unpack_dequant(card2, d)
    assert np.array_equal(k3[:, :, t16], K.view(np.uint16)[:, :, t16])


def test_uniform_cards_and_group_sizes():
    for G in (32, 64, 128):
        for w in (2, 4, 8):
            L, H, T, D = 1, 1, 33, 128
            K, V = qkv_synth.make_kv(L, H, T, D, 5, "llama")
            d = ref.make_desc(L, H, T, D, G)
            bits = np.full(T, w, dtype=np.uint8)
            counts = [T if x == w else 0 for x in WIDTHS]
            card = ref.quantize_pack(d, K.numpy(), V.numpy(), bits, counts)
            assert card.shape[0] == layout(L, H, T, D, G, counts)["total"]
            k2, _ = ref.unpack_dequant(card, d)
            # compare one row against the single-group functions
            row = K.numpy().view(np.uint16)[0, 0, 17]
            want = []
            for g in range(D // G):
                sh, zh, q = ref.quantize_group(row[g * G:(g + 1) * G], w)
                want.append(ref.dequantize_group(q, sh, zh))
            assert np.array_equal(k2[0, 0, 17], np.concatenate(want))


def test_pack_and_unpack_reject_bad_input():
    d, K, V, bits = tiny_problem()
    counts = ref.count_bits(bits)
    with pytest.raises(ref.OracleError):
        ref.quantize_pack(d, K, V, bits, counts, capacity=ref.card_bytes(d, counts) - 1)
    wrong = counts.copy(); wrong[0] += 1; wrong[1] -= 1
    with pytest.raises(ref.OracleError):
        ref.quantize_pack(d, K, V, bits, wrong)
    bad = bits.copy(); bad[3] = 5
    with pytest.raises(ref.OracleError):
        ref.quantize_pack(d, K, V, bad, counts)
    card = ref.quantize_pack(d, K, V, bits, counts)
    with pytest.raises(ref.OracleError):
        ref.unpack_dequant(card[:-1], d)                       # truncated
    broken = card.copy(); broken[0] ^= 1
    with pytest.raises(ref.OracleError):
        ref.unpack_dequant(broken, d)                          # bad magic
    other = ref.make_desc(d.layers, d.kv_heads, d.tokens + 1, d.head_dim, d.group_size)
    with pytest.raises(ref.OracleError):
        ref.unpack_dequant(card, other)                        # shape mismatch
    dd, cc, avg, status = ref.card_peek(card)
    assert (dd.layers, dd.kv_heads, dd.tokens, dd.head_dim, dd.group_size) == (1, 2, 96, 128, 32)
    assert cc.tolist() == counts.tolist() and status == 0


def test_unpack_refuses_a_card_whose_tables_disagree():
    """bits, slot and order must tell one story (order the inverse of slot, slot the stable rank); the oracle
    refuses the whole card when any of them is touched, and accepts it again when the damage is undone."""
    d, K, V, bits = tiny_problem()
    counts = ref.count_bits(bits)
    card = ref.quantize_pack(d, K, V, bits, counts)
    off = ref.card_offsets(d, counts)
    T = d.tokens

    def entry(table, i):
        return slice(off[table] + 4 * i, off[table] + 4 * i + 4)

    def refused(c):
        with pytest.raises(ref.OracleError) as e:
            ref.unpack_dequant(c, d)
        return e.value.code == -9

    order = card[off["order"]:off["order"] + 4 * T].view(np.uint32)
    assert sorted(order.tolist()) == list(range(T))
    dup = card.copy(); dup[entry("order", 5)] = card[entry("order", 6)]                      # a token named twice
    far = card.copy(); far[entry("order", 5)] = np.frombuffer((T + 7).to_bytes(4, "little"), dtype=np.uint8)
    swap = card.copy(); swap[entry("order", 0)] = card[entry("order", T - 1)]; swap[entry("order", T - 1)] = card[entry("order", 0)]
    slot = card.copy(); slot[entry("slot", 9)] = np.frombuffer((3).to_bytes(4, "little"), dtype=np.uint8) if \
        int.from_bytes(card[entry("slot", 9)].tobytes(), "little") != 3 else np.frombuffer((4).to_bytes(4, "little"), dtype=np.uint8)
    width = card.copy(); width[off["bits"] + 2] = 2 if bits[2] != 2 else 4                     # a token moved to another class
    for broken in (dup, far, swap, slot, width):
        assert refused(broken)
    ref.unpack_dequant(card, d)                                                                 # the untouched card still unpacks


def test_generator_is_reproducible_and_device_free():
    a = qkv_synth.make_kv(1, 2, 64, 128, 1001, "tiny")
    b = qkv_synth.make_kv(1, 2, 64, 128, 1001, "tiny")
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    c = qkv_synth.make_kv(1, 2, 64, 128, 1002, "tiny")
    assert not torch.equal(a[0], c[0])
    assert torch.isfinite(a[0].float()).all()
