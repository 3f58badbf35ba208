"""GPU parity of the one-launch path from scores to a planned card (qkv_assign_plan,
qkv_assign_quantize_pack) against the CPU oracle, and the bounds qkv_card_fill keeps on a card
whose tables it cannot trust.

Bar: widths, class counts, header, bits / slot / order tables, pads and - for the whole-card
call - every code, pair and raw row byte-identical to the oracle's rank-quantile allocator
followed by its compaction and quantizer on the same seeded inputs.
"""
import numpy as np
import pytest
import torch

import paper_2605_03884_amd as qkv
import qkv_synth
from oracle import ref

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
BUDGETS = (2.0, 2.001, 3.0, 4.0, 5.0, 7.5, 15.999, 16.0)


def say(msg):
    print("[case] " + msg, flush=True)


def score_variants(T, rng):
    return {
        "uniform": rng.random(T).astype(np.float32),
        "ties": (np.round(rng.random(T) * 7) / 7).astype(np.float32),
        "all equal": np.full(T, 0.25, dtype=np.float32),
        "signed": rng.standard_normal(T).astype(np.float32),
        "zeros": rng.choice(np.array([0.0, -0.0, 1e-40, -1e-40], dtype=np.float32), size=T),
        "sorted": np.sort(rng.random(T).astype(np.float32)),
        "infs": rng.choice(np.array([np.inf, -np.inf, 0.0, 1.0], dtype=np.float32), size=T),
    }


def oracle_front_matter(desc, bits, counts):
    """Header, tables and pads as the oracle writes them: the front of the card of an all-zero cache."""
    rd = ref.make_desc(desc.layers, desc.kv_heads, desc.tokens, desc.head_dim, desc.group_size, desc.model_id,
                       desc.sender_id, desc.position_offset)
    zeros = np.zeros((desc.layers, desc.kv_heads, desc.tokens, desc.head_dim), dtype=np.uint16)
    card = ref.quantize_pack(rd, zeros, zeros, bits, counts)
    return card[:ref.card_offsets(rd, counts)["codes2"]], card.size


@pytest.mark.parametrize("T", [1, 2, 7, 8, 63, 64, 1000, 1024, 4097, 8191, 8192, 8193, 20001, 32768, 32769, 100003])
def test_assign_plan_matches_oracle(T):
    say("assign_plan T=%d" % T)
    rng = np.random.default_rng(1000 + T)
    desc = qkv.Desc.make(1, 1, T, 64, 32, model_id=0xABCDEF0123, sender_id=T, position_offset=-17)
    for name, scores in score_variants(T, rng).items():
        sd = torch.from_numpy(scores).to(DEV)
        for budget in BUDGETS:
            wb, wc = ref.assign_bits(scores, budget)
            slot, order, _ = ref.compact(wb)
            front, total = oracle_front_matter(desc, wb, wc)
            assert qkv.card_bytes(desc, wc.tolist()) == total
            card = torch.full((total + 256,), 0xA5, dtype=torch.uint8, device=DEV)
            bits = torch.full((T + 8,), 0x5A, dtype=torch.uint8, device=DEV)
            counts = qkv.assign_plan(desc, sd, budget, card[:total], bits=bits[:T])
            torch.cuda.synchronize()
            assert counts == wc.tolist(), (name, budget)
            got = card.cpu().numpy()
            assert np.array_equal(bits.cpu().numpy()[:T], wb), (name, budget)
            assert np.all(bits.cpu().numpy()[T:] == 0x5A)
            assert np.all(got[total:] == 0xA5), "bytes behind the card were written"
            bad = np.flatnonzero(got[:front.size] != front)
            assert bad.size == 0, (name, budget, int(bad[0]), int(got[bad[0]]), int(front[bad[0]]))
            off = ref.card_offsets(ref.make_desc(1, 1, T, 64, 32), wc)
            assert np.array_equal(got[off["slot"]:off["slot"] + 4 * T].view(np.uint32), slot)
            assert np.array_equal(got[off["order"]:off["order"] + 4 * T].view(np.uint32), order)


def test_assign_plan_equals_assign_then_plan_and_takes_no_bits_pointer():
    rng = np.random.default_rng(5)
    for T in (300, 8192, 9000, 40000):
        desc = qkv.Desc.make(2, 2, T, 128, 64, model_id=9, sender_id=4)
        scores = torch.from_numpy(rng.random(T).astype(np.float32)).to(DEV)
        for budget in (2.5, 6.0):
            bits, counts = qkv.assign_bits(scores, budget)
            n = qkv.card_bytes(desc, counts)
            a = torch.full((n,), 0xA5, dtype=torch.uint8, device=DEV)
            b = torch.full((n,), 0xA5, dtype=torch.uint8, device=DEV)
            qkv.card_plan(desc, bits, counts, a)
            assert qkv.assign_plan(desc, scores, budget, b) == counts          # bits=None
            torch.cuda.synchronize()
            assert torch.equal(a, b)


def test_unaligned_scores_and_bits_pointers():
    T = 5000
    rng = np.random.default_rng(6)
    desc = qkv.Desc.make(1, 1, T, 64, 32)
    base_s = torch.zeros(T + 4, dtype=torch.float32, device=DEV)
    base_b = torch.zeros(T + 16, dtype=torch.uint8, device=DEV)
    scores = rng.random(T).astype(np.float32)
    for so in (0, 1, 3):
        for bo in (0, 1, 5):
            base_s[so:so + T].copy_(torch.from_numpy(scores))
            wb, wc = ref.assign_bits(scores, 4.0)
            card = torch.zeros(qkv.card_bytes(desc, wc.tolist()), dtype=torch.uint8, device=DEV)
            qkv.assign_plan(desc, base_s[so:so + T], 4.0, card, bits=base_b[bo:bo + T])
            torch.cuda.synchronize()
            assert np.array_equal(base_b[bo:bo + T].cpu().numpy(), wb)
            front, _ = oracle_front_matter(desc, wb, wc)
            assert np.array_equal(card.cpu().numpy()[:front.size], front)


@pytest.mark.parametrize("L,H,T,D,G,budget", [(2, 2, 300, 128, 32, 4.0), (1, 3, 2500, 64, 32, 3.0), (2, 1, 9001, 128, 64, 6.5),
                                              (1, 1, 33000, 256, 128, 2.7)])
def test_assign_quantize_pack_whole_card(L, H, T, D, G, budget):
    say("assign_quantize_pack L=%d H=%d T=%d D=%d G=%d B=%s" % (L, H, T, D, G, budget))
    K, V = qkv_synth.make_kv(L, H, T, D, 7000 + T, "llama")
    scores = qkv_synth.make_scores(T, 7001 + T)
    desc = qkv.Desc.make(L, H, T, D, G, model_id=77, sender_id=5, position_offset=12)
    wb, wc = ref.assign_bits(scores.numpy(), budget)
    rd = ref.make_desc(L, H, T, D, G, 77, 5, 12)
    want = ref.quantize_pack(rd, K.numpy(), V.numpy(), wb, wc)
    card = torch.full((want.size + 512,), 0xA5, dtype=torch.uint8, device=DEV)
    bits = torch.empty(T, dtype=torch.uint8, device=DEV)
    counts = qkv.assign_quantize_pack(desc, K.to(DEV), V.to(DEV), scores.to(DEV), budget, card[:want.size], bits=bits)
    torch.cuda.synchronize()
    got = card.cpu().numpy()
    assert counts == wc.tolist()
    assert np.array_equal(bits.cpu().numpy(), wb)
    assert np.all(got[want.size:] == 0xA5)
    bad = np.flatnonzero(got[:want.size] != want)
    assert bad.size == 0, (int(bad[0]), int(bad.size))
    _, c2, _, status = qkv.card_peek(card, card_nbytes=want.size)
    assert status == 0 and c2 == counts


def test_assign_plan_host_errors():
    T = 100
    desc = qkv.Desc.make(1, 1, T, 64, 32)
    scores = torch.zeros(T, dtype=torch.float32, device=DEV)
    n = qkv.card_bytes(desc, qkv.budget_counts(T, 4.0))
    card = torch.zeros(n + 256, dtype=torch.uint8, device=DEV)
    for budget in (1.9, 16.5, float("nan")):
        with pytest.raises(qkv.QkvError) as e:
            qkv.assign_plan(desc, scores, budget, card)
        assert e.value.code == -4
    with pytest.raises(qkv.QkvError) as e:
        qkv.assign_plan(desc, scores, 4.0, card[:n - 1])
    assert e.value.code == -5
    with pytest.raises(qkv.QkvError) as e:
        qkv.assign_plan(desc, scores, 4.0, card[1:])
    assert e.value.code == -6
    with pytest.raises(qkv.QkvError) as e:
        qkv.assign_plan(qkv.Desc.make(1, 1, T, 96, 32), scores, 4.0, card)
    assert e.value.code == -2
    assert torch.all(card == 0)                         # nothing was written on any error


# ------------------------------------------------------------------ a card whose tables cannot be trusted


def fenced(t, fill):
    """A copy of tensor t inside a larger allocation with 4096 canary bytes on either side."""
    raw = torch.full((t.numel() * t.element_size() + 8192,), fill, dtype=torch.uint8, device=DEV)
    inner = raw[4096:4096 + t.numel() * t.element_size()].view(t.dtype).view(t.shape)
    inner.copy_(t)
    return raw, inner


def test_card_fill_on_a_card_that_was_never_planned_stays_in_bounds():
    L, H, T, D, G = 2, 2, 700, 128, 32
    K, V = qkv_synth.make_kv(L, H, T, D, 801, "llama")
    desc = qkv.Desc.make(L, H, T, D, G)
    counts = [300, 200, 150, 50]
    n = qkv.card_bytes(desc, counts)
    k_raw, Kd = fenced(K.to(DEV), 0x3C)
    v_raw, Vd = fenced(V.to(DEV), 0x3C)
    card = torch.full((n + 4096,), 0xA5, dtype=torch.uint8, device=DEV)       # every order[] entry reads 0xA5A5A5A5
    say("card_fill on 0xA5 bytes")
    qkv.card_fill(desc, Kd, Vd, counts, card[:n])
    torch.cuda.synchronize()
    got = card.cpu().numpy()
    assert np.all(got[n:] == 0xA5), "bytes behind the card were written"
    for raw in (k_raw, v_raw):
        h = raw.cpu().numpy()
        assert np.all(h[:4096] == 0x3C) and np.all(h[-4096:] == 0x3C)
    assert torch.equal(Kd.cpu(), K) and torch.equal(Vd.cpu(), V)
    status = int(got[192:196].view(np.uint32)[0])
    assert status & qkv.STATUS_BAD_ORDER
    assert status | qkv.STATUS_BAD_ORDER == 0xA5A5A5A5 | qkv.STATUS_BAD_ORDER   # nothing else in the header was touched
    with pytest.raises(qkv.QkvError) as e:
        qkv.card_peek(card, card_nbytes=n)
    assert e.value.code == -9
    # no token was found, so every row was made from zeros: all codes, pairs and raw rows are zero
    # (the pads behind the sections belong to the planning step and keep their 0xA5)
    off = ref.card_offsets(ref.make_desc(L, H, T, D, G), counts)
    P = 2 * L * H
    for c, w in enumerate((2, 4, 8)):
        codes, pairs = P * counts[c] * D * w // 8, P * counts[c] * (D // G) * 4
        assert not got[off["codes%d" % w]:off["codes%d" % w] + codes].any()
        assert not got[off["meta%d" % w]:off["meta%d" % w] + pairs].any()
    assert not got[off["fp16"]:off["fp16"] + P * counts[3] * D * 2].any()


def test_card_fill_skips_an_order_entry_that_names_no_token():
    L, H, T, D, G = 1, 2, 333, 128, 32
    K, V = qkv_synth.make_kv(L, H, T, D, 811, "llama")
    bits = qkv_synth.make_bits_uniform_choice(T, 812).numpy()
    counts = [int((bits == w).sum()) for w in (2, 4, 8, 16)]
    desc = qkv.Desc.make(L, H, T, D, G)
    rd = ref.make_desc(L, H, T, D, G)
    want = ref.quantize_pack(rd, K.numpy(), V.numpy(), bits, counts)
    off = ref.card_offsets(rd, counts)
    Kd, Vd, bd = K.to(DEV), V.to(DEV), torch.from_numpy(bits).to(DEV)
    card = torch.zeros(want.size, dtype=torch.uint8, device=DEV)
    qkv.card_plan(desc, bd, counts, card)
    j = counts[0] + 3                                   # row 3 of the 4-bit segment
    card[off["order"] + 4 * j:off["order"] + 4 * j + 4] = torch.tensor([0xFF, 0xFF, 0xFF, 0x7F], dtype=torch.uint8)
    qkv.card_fill(desc, Kd, Vd, counts, card)
    torch.cuda.synchronize()
    got = card.cpu().numpy()
    assert qkv.card_peek(card)[3] == qkv.STATUS_BAD_ORDER
    # the card equals the oracle's except for the status word, the planted entry, and that row in every plane (zeros)
    mask = np.ones(want.size, dtype=bool)
    mask[192:196] = False
    mask[off["order"] + 4 * j:off["order"] + 4 * j + 4] = False
    n4 = counts[1]
    for p in range(2 * L * H):
        r = p * n4 + 3
        c0, m0 = off["codes4"] + r * (D // 2), off["meta4"] + r * (D // G) * 4
        mask[c0:c0 + D // 2] = False
        mask[m0:m0 + (D // G) * 4] = False
        assert not got[c0:c0 + D // 2].any() and not got[m0:m0 + (D // G) * 4].any()
    assert np.array_equal(got[mask], want[mask])
