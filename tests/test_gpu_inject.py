"""GPU parity of the injection into per-layer caches (layer ranges, strides, prefix) with optional
rotary realignment of the keys, through the C ABI, against the CPU oracle.  Bar: every fp16 value
bit-identical (both sides take the same roundings), nothing outside the injected rows touched."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2605_03884_amd as qkv
import qkv_synth
from oracle import inject_ref, ref

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
CANARY = 0x7E11           # a NaN pattern no dequantized value has


def say(msg):
    print("[case] " + msg, flush=True)


def make_card(L, H, T, D, G, seed, bits=None, kind="llama"):
    K, V = qkv_synth.make_kv(L, H, T, D, seed, kind)
    if bits is None:
        bits = qkv_synth.make_bits_uniform_choice(T, seed + 1).numpy()
    counts = ref.count_bits(bits).tolist()
    desc = qkv.Desc.make(L, H, T, D, G, model_id=3, sender_id=4, position_offset=11)
    card = torch.empty(qkv.card_bytes(desc, counts), dtype=torch.uint8, device=DEV)
    qkv.quantize_pack(desc, K.to(DEV), V.to(DEV), torch.from_numpy(bits).to(DEV), counts, card)
    torch.cuda.synchronize()
    rdesc = ref.make_desc(L, H, T, D, G, 3, 4, 11)
    return desc, rdesc, card, card.cpu().numpy()


def caches(n, H, cap, D):
    mk = lambda: torch.full((H, cap, D), 0, dtype=torch.int16, device=DEV).fill_(CANARY).view(torch.float16)
    return [mk() for _ in range(n)], [mk() for _ in range(n)]


def host_caches(n, H, cap, D):
    return ([np.full((H, cap, D), CANARY, np.uint16) for _ in range(n)], [np.full((H, cap, D), CANARY, np.uint16) for _ in range(n)])


def check(desc, rdesc, card, card_host, layer_begin, count, cap, prefix, rope, label):
    say(label)
    H, T, D = desc.kv_heads, desc.tokens, desc.head_dim
    kc, vc = caches(count, H, cap, D)
    status = torch.full((1,), 0x7777, dtype=torch.int32, device=DEV)
    qkv.inject_layers(card, desc, [k[:, prefix:prefix + T] for k in kc], [v[:, prefix:prefix + T] for v in vc],
                      layer_begin, rope_base=rope[0] if rope else 0.0, rope_delta=rope[1] if rope else 0, status=status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    wk, wv = host_caches(count, H, cap, D)
    inject_ref.inject_layers(card_host, rdesc, wk, wv, layer_begin, prefix, rope)
    for i in range(count):
        gk = kc[i].view(torch.int16).cpu().numpy().view(np.uint16)
        gv = vc[i].view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(gv, wv[i]), (label, "V layer", i)
        if not np.array_equal(gk, wk[i]):
            idx = np.argwhere(gk != wk[i])[0]
            raise AssertionError((label, "K layer", i, idx.tolist(), hex(gk[tuple(idx)]), hex(wk[i][tuple(idx)]),
                                  int((gk != wk[i]).sum())))


@pytest.mark.parametrize("G", [32, 64, 128])
def test_all_layers_no_realignment_equals_dense_unpack(G):
    desc, rdesc, card, host = make_card(3, 2, 300, 128, G, 40 + G)
    check(desc, rdesc, card, host, 0, 3, 300, 0, None, "inject all layers G=%d" % G)


@pytest.mark.parametrize("D,G", [(64, 32), (128, 32), (128, 64), (256, 128), (256, 32)])
def test_realignment_every_head_dim(D, G):
    desc, rdesc, card, host = make_card(2, 3, 333, D, G, 50 + D + G)
    check(desc, rdesc, card, host, 0, 2, 333 + 20, 7, (10000.0, 37), "inject rope D=%d G=%d" % (D, G))


@pytest.mark.parametrize("rope", [(10000.0, 1), (500000.0, 4096), (10000.0, -123), (1000000.0, 131072), (10000.0, 0), (2.0, 3)])
def test_realignment_bases_and_shifts(rope):
    desc, rdesc, card, host = make_card(2, 2, 257, 128, 32, 61)
    check(desc, rdesc, card, host, 0, 2, 400, 100, rope, "inject rope %s" % (rope,))


def test_layer_ranges_and_untouched_neighbours():
    L = 7
    desc, rdesc, card, host = make_card(L, 2, 200, 128, 32, 71)
    for lb, n in ((0, 1), (3, 1), (6, 1), (2, 3), (0, 7), (5, 2)):
        check(desc, rdesc, card, host, lb, n, 256, 16, (10000.0, 5), "inject layers [%d, %d)" % (lb, lb + n))


@pytest.mark.parametrize("width", [2, 4, 8, 16])
def test_uniform_cards(width):
    T = 500
    bits = np.full(T, width, np.uint8)
    desc, rdesc, card, host = make_card(2, 2, T, 128, 32, 80 + width, bits=bits)
    check(desc, rdesc, card, host, 0, 2, T, 0, (10000.0, 77), "inject uniform %d-bit" % width)
    check(desc, rdesc, card, host, 1, 1, T + 8, 8, None, "inject uniform %d-bit, no rope" % width)


def test_skewed_mix_long_sequence():
    T = 5000
    scores = qkv_synth.make_scores(T, 91).numpy()
    bits, _ = ref.assign_bits(scores, 3.0)
    desc, rdesc, card, host = make_card(2, 4, T, 128, 32, 92, bits=bits)
    check(desc, rdesc, card, host, 0, 2, T + 64, 64, (500000.0, 1000), "inject 5000 tokens, budget 3")


def test_one_token_and_tiny_shapes():
    for T in (1, 2, 31, 33):
        desc, rdesc, card, host = make_card(1, 1, T, 128, 32, 100 + T)
        check(desc, rdesc, card, host, 0, 1, T + 3, 3, (10000.0, 9), "inject T=%d" % T)


def test_layer_at_a_time_on_two_streams_equals_one_call():
    say("inject layer by layer on two streams")
    L, H, T, D = 6, 2, 700, 128
    desc, rdesc, card, host = make_card(L, H, T, D, 32, 111)
    kc, vc = caches(L, H, T, D)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    done = []
    torch.cuda.synchronize()
    for l in range(L):
        s = streams[l % 2]
        with torch.cuda.stream(s):
            qkv.inject_layers(card, desc, [kc[l]], [vc[l]], l, rope_base=10000.0, rope_delta=50)
            e = torch.cuda.Event()
            e.record(s)
            done.append(e)
    for e in done:
        e.synchronize()
    k1, v1 = caches(L, H, T, D)
    qkv.inject_layers(card, desc, k1, v1, 0, rope_base=10000.0, rope_delta=50)
    torch.cuda.synchronize()
    for l in range(L):
        assert torch.equal(kc[l].view(torch.int16), k1[l].view(torch.int16))
        assert torch.equal(vc[l].view(torch.int16), v1[l].view(torch.int16))


def test_sixty_four_layers_in_one_call():
    L = 64
    desc, rdesc, card, host = make_card(L, 1, 70, 128, 32, 121)
    check(desc, rdesc, card, host, 0, 64, 70, 0, (10000.0, 3), "inject 64 layers")


def test_corrupt_cards_write_nothing_or_stay_in_bounds():
    say("inject corrupt cards")
    desc, rdesc, card, host = make_card(2, 2, 300, 128, 32, 131)
    kc, vc = caches(2, 2, 300, 128)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    bad = card.clone()
    bad[0] = 0                                                   # magic
    qkv.inject_layers(bad, desc, kc, vc, 0, rope_base=10000.0, rope_delta=1, status=status)
    torch.cuda.synchronize()
    assert int(status.item()) == qkv.STATUS_BAD_HEADER
    for t in kc + vc:
        assert bool((t.view(torch.int16) == CANARY).all())
    # order entries out of range: flagged, the rows skipped, everything else as before
    off = ref.card_offsets(rdesc, ref.count_bits(host[256:256 + 300]).tolist())
    bad = card.clone()
    o = bad[off["order"]:off["order"] + 4 * 300].view(torch.int32)
    victims = [0, 150, 299]
    lost = [int(o[v].item()) for v in victims]
    for v in victims:
        o[v] = 300 + v
    status.zero_()
    qkv.inject_layers(bad, desc, kc, vc, 0, status=status)
    torch.cuda.synchronize()
    assert int(status.item()) == qkv.STATUS_BAD_ORDER
    wk, wv = host_caches(2, 2, 300, 128)
    inject_ref.inject_layers(host, rdesc, wk, wv, 0, 0)
    for i in range(2):
        gk = kc[i].view(torch.int16).cpu().numpy().view(np.uint16)
        keep = np.ones(300, bool)
        keep[lost] = False
        assert np.array_equal(gk[:, keep], wk[i][:, keep])
        assert np.all(gk[:, lost] == CANARY)


def test_inject_host_errors():
    desc, rdesc, card, host = make_card(4, 2, 64, 128, 32, 141)
    kc, vc = caches(4, 2, 64, 128)
    L = qkv.lib()

    def call(lb, n, hs=64 * 128, ts=128, base=0.0, delta=0, kptrs=None, card_ptr=None, nbytes=None, per_channel=0):
        kp = (ctypes.c_void_p * max(n, 1))(*(kptrs if kptrs is not None else [kc[i % 4].data_ptr() for i in range(max(n, 1))]))
        vp = (ctypes.c_void_p * max(n, 1))(*[vc[i % 4].data_ptr() for i in range(max(n, 1))])
        w = qkv.Inject(lb, n, kp, vp, hs, ts, base, delta, per_channel, 0)
        return L.qkv_inject_layers(card.data_ptr() if card_ptr is None else card_ptr, card.numel() if nbytes is None else nbytes,
                                   ctypes.byref(desc), ctypes.byref(w), None, None)

    assert call(0, 4) == 0
    assert call(0, 0) == -2 and call(-1, 1) == -2 and call(3, 2) == -2 and call(0, 65) == -2
    assert call(0, 1, ts=120) == -2 and call(0, 1, ts=132) == -2 and call(0, 1, hs=4) == -2
    assert call(0, 1, base=-1.0) == -2 and call(0, 1, base=float("nan")) == -2 and call(0, 1, base=1e4, delta=1 << 31) == -2
    assert call(0, 1, kptrs=[kc[0].data_ptr() + 2]) == -6
    assert call(0, 1, kptrs=[None]) == -1
    assert call(0, 1, card_ptr=card.data_ptr() + 16) == -6
    assert call(0, 1, nbytes=100) == -5
    assert call(0, 1, per_channel=2) == -2
    assert call(0, 1, per_channel=1) == 0                 # shape fits the per-channel rules; the device refuses the card's grouping
    assert L.qkv_inject_layers(card.data_ptr(), card.numel(), ctypes.byref(desc), None, None, None) == -1
    # strides that would carry a row address out of range for the shape are refused before anything is launched
    huge = qkv.Desc.make(1, 1, 1 << 30, 128, 32)
    kp = (ctypes.c_void_p * 1)(kc[0].data_ptr())
    vp = (ctypes.c_void_p * 1)(vc[0].data_ptr())
    w = qkv.Inject(0, 1, kp, vp, 1 << 20, 1 << 20, 0.0, 0, 0, 0)
    assert L.qkv_inject_layers(card.data_ptr(), card.numel(), ctypes.byref(huge), ctypes.byref(w), None, None) == -2
    torch.cuda.synchronize()


def test_random_shapes_ranges_and_shifts():
    rng = np.random.default_rng(2024)
    for case in range(24):
        D = int(rng.choice([64, 128, 256]))
        G = int(rng.choice([g for g in (32, 64, 128) if g <= D]))
        L = int(rng.integers(1, 6))
        H = int(rng.integers(1, 5))
        T = int(rng.integers(1, 700))
        lb = int(rng.integers(0, L))
        n = int(rng.integers(1, L - lb + 1))
        prefix = int(rng.integers(0, 50))
        cap = prefix + T + int(rng.integers(0, 30))
        rope = None if case % 3 == 0 else (float(rng.choice([10000.0, 500000.0, 1e6])), int(rng.integers(-5000, 100000)))
        kind = ["choice", "budget", "uniform"][case % 3]
        if kind == "choice":
            bits = qkv_synth.make_bits_uniform_choice(T, 3000 + case).numpy()
        elif kind == "budget":
            bits, _ = ref.assign_bits(qkv_synth.make_scores(T, 3100 + case).numpy(), float(rng.choice([2.5, 3.0, 5.0, 9.0])))
        else:
            bits = np.full(T, int(rng.choice([2, 4, 8, 16])), np.uint8)
        desc, rdesc, card, host = make_card(L, H, T, D, G, 3200 + case, bits=bits)
        check(desc, rdesc, card, host, lb, n, cap, prefix, rope,
              "inject random %d: L=%d H=%d T=%d D=%d G=%d layers [%d,%d) prefix=%d rope=%s %s"
              % (case, L, H, T, D, G, lb, lb + n, prefix, rope, kind))
