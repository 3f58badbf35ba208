"""GPU parity of the card variant with keys grouped per channel (uniform cards): qkv_quantize_pack_kc and
qkv_unpack_dequant_kc through the C ABI against the CPU oracle, every card byte and every fp16 value."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2605_03884_amd as qkv
import qkv_synth
from oracle import ref

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
CLASS = {2: 0, 4: 1, 8: 2}


def say(msg):
    print("[case] " + msg, flush=True)


def problem(L, H, T, D, width, seed, kind="llama"):
    K, V = qkv_synth.make_kv(L, H, T, D, seed, kind)
    bits = np.full(T, width, np.uint8)
    counts = [0, 0, 0, 0]
    counts[CLASS[width]] = T
    desc = qkv.Desc.make(L, H, T, D, 32, model_id=9, sender_id=8, position_offset=3)
    rdesc = ref.make_desc(L, H, T, D, 32, 9, 8, 3)
    return K, V, bits, counts, desc, rdesc


def run(L, H, T, D, width, seed, label):
    say(label)
    K, V, bits, counts, desc, rdesc = problem(L, H, T, D, width, seed)
    n = qkv.card_bytes(desc, counts)
    card = torch.full((n + 512,), 0xA5, dtype=torch.uint8, device=DEV)
    qkv.quantize_pack_kc(desc, K.to(DEV), V.to(DEV), torch.from_numpy(bits).to(DEV), counts, card[:n])
    torch.cuda.synchronize()
    want = ref.quantize_pack_kc(rdesc, K.numpy().view(np.uint16), V.numpy().view(np.uint16), bits, counts)
    got = card.cpu().numpy()
    assert np.all(got[n:] == 0xA5)
    diff = np.flatnonzero(got[:n] != want)
    assert diff.size == 0, (label, "card differs at %d bytes, first %d" % (diff.size, int(diff[0])))
    shape = (L, H, T, D)
    ko = torch.full(shape, float("nan"), dtype=torch.float16, device=DEV)
    vo = torch.full(shape, float("nan"), dtype=torch.float16, device=DEV)
    status = torch.full((1,), 0x7777, dtype=torch.int32, device=DEV)
    qkv.unpack_dequant_kc(card[:n], desc, ko, vo, status=status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    wk, wv = ref.unpack_dequant_kc(want, rdesc)
    assert np.array_equal(ko.cpu().numpy().view(np.uint16), wk), label
    assert np.array_equal(vo.cpu().numpy().view(np.uint16), wv), label
    d2, c2, avg, st = qkv.card_peek(card[:n])
    assert st == 0 and c2 == counts and abs(avg - width) < 1e-6
    return card[:n], desc, rdesc, K, V


@pytest.mark.parametrize("width", [2, 4, 8])
@pytest.mark.parametrize("D,T", [(128, 32), (128, 96), (128, 1056), (64, 64), (64, 192), (64, 1088)])
def test_card_and_cache_match_oracle(width, D, T):
    run(2, 3, T, D, width, 10 * width + D + T, "kc width=%d D=%d T=%d" % (width, D, T))


def test_single_plane_and_many_planes():
    run(1, 1, 64, 128, 4, 71, "kc one plane")
    run(5, 7, 160, 128, 2, 72, "kc 35 planes")


def test_tiny_kind_and_special_values():
    say("kc special values")
    L, H, T, D = 1, 2, 128, 128
    K, V, bits, counts, desc, rdesc = problem(L, H, T, D, 4, 81, kind="tiny")
    Kn = K.numpy().copy()
    Kn[0, 0, :32, 5] = 0.0                          # a constant channel block: scale 0
    Kn[0, 0, 32:64, 6] = np.float16(6e-8)           # subnormals
    Kn[0, 1, :32, 7] = np.linspace(-60000, 60000, 32).astype(np.float16)     # the widest range
    Kn[0, 1, 64:96, 9] = np.where(np.arange(32) % 2 == 0, np.float16(-0.0), np.float16(0.0))
    K = torch.from_numpy(Kn)
    n = qkv.card_bytes(desc, counts)
    card = torch.empty(n, dtype=torch.uint8, device=DEV)
    qkv.quantize_pack_kc(desc, K.to(DEV), V.to(DEV), torch.from_numpy(bits).to(DEV), counts, card)
    torch.cuda.synchronize()
    want = ref.quantize_pack_kc(rdesc, Kn.view(np.uint16), V.numpy().view(np.uint16), bits, counts)
    assert np.array_equal(card.cpu().numpy(), want)
    ko = torch.empty((L, H, T, D), dtype=torch.float16, device=DEV)
    vo = torch.empty_like(ko)
    qkv.unpack_dequant_kc(card, desc, ko, vo)
    torch.cuda.synchronize()
    wk, wv = ref.unpack_dequant_kc(want, rdesc)
    assert np.array_equal(ko.cpu().numpy().view(np.uint16), wk) and np.array_equal(vo.cpu().numpy().view(np.uint16), wv)


def test_the_two_groupings_refuse_each_other_on_the_device():
    say("kc mutual refusal")
    card_kc, desc, rdesc, K, V = run(2, 2, 128, 128, 4, 91, "kc card for refusal")
    shape = (2, 2, 128, 128)
    canary = 0x7E11
    mk = lambda: torch.zeros(shape, dtype=torch.int16, device=DEV).fill_(canary).view(torch.float16)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    ko, vo = mk(), mk()
    qkv.unpack_dequant(card_kc, desc, ko, vo, status=status)              # per-token call on a per-channel card
    torch.cuda.synchronize()
    assert int(status.item()) == qkv.STATUS_BAD_HEADER
    assert bool((ko.view(torch.int16) == canary).all()) and bool((vo.view(torch.int16) == canary).all())
    counts = [0, 128, 0, 0]
    card_pt = torch.empty(qkv.card_bytes(desc, counts), dtype=torch.uint8, device=DEV)
    bits = torch.full((128,), 4, dtype=torch.uint8, device=DEV)
    qkv.quantize_pack(desc, K.to(DEV), V.to(DEV), bits, counts, card_pt)
    status.zero_()
    qkv.unpack_dequant_kc(card_pt, desc, ko, vo, status=status)           # per-channel call on a per-token card
    torch.cuda.synchronize()
    assert int(status.item()) == qkv.STATUS_BAD_HEADER
    assert bool((ko.view(torch.int16) == canary).all()) and bool((vo.view(torch.int16) == canary).all())
    # the header says which grouping a card has
    assert qkv.card_flags(card_kc) == qkv.FLAG_KEYS_PER_CHANNEL and qkv.card_flags(card_pt) == 0
    broken = card_kc.clone()
    broken[188] = 3                                                        # an unknown flag bit
    with pytest.raises(qkv.QkvError) as err:
        qkv.card_flags(broken)
    assert err.value.code == -9
    with pytest.raises(qkv.QkvError):
        qkv.card_peek(broken)
    # injection must be told the grouping; attention reads per-token groups only
    status.zero_()
    qkv.inject_layers(card_kc, desc, [ko[0], ko[1]], [vo[0], vo[1]], 0, status=status)
    torch.cuda.synchronize()
    assert int(status.item()) == qkv.STATUS_BAD_HEADER and bool((ko.view(torch.int16) == canary).all())
    status.zero_()
    qkv.inject_layers(card_pt, desc, [ko[0], ko[1]], [vo[0], vo[1]], 0, status=status, keys_per_channel=True)
    torch.cuda.synchronize()
    assert int(status.item()) == qkv.STATUS_BAD_HEADER and bool((ko.view(torch.int16) == canary).all())
    q = torch.zeros((2, 8, 128), dtype=torch.float16, device=DEV)
    out = torch.full((2, 8, 128), 7.0, dtype=torch.float32, device=DEV)
    status.zero_()
    qkv.card_attend(card_kc, desc, q, 0.1, out, status=status)
    torch.cuda.synchronize()
    assert int(status.item()) == qkv.STATUS_BAD_HEADER and bool((out == 7.0).all())


def test_kc_host_errors():
    L = qkv.lib()
    K = torch.zeros((1, 1, 64, 128), dtype=torch.float16, device=DEV)
    bits = torch.full((64,), 4, dtype=torch.uint8, device=DEV)
    card = torch.empty(1 << 20, dtype=torch.uint8, device=DEV)

    def pack(desc, counts):
        c = (ctypes.c_int64 * 4)(*counts)
        return L.qkv_quantize_pack_kc(ctypes.byref(desc), K.data_ptr(), K.data_ptr(), bits.data_ptr(), c, card.data_ptr(),
                                      card.numel(), None)

    assert pack(qkv.Desc.make(1, 1, 64, 128, 32), [0, 64, 0, 0]) == 0
    assert pack(qkv.Desc.make(1, 1, 64, 128, 64), [0, 64, 0, 0]) == -2          # group size
    assert pack(qkv.Desc.make(1, 1, 48, 128, 32), [0, 48, 0, 0]) == -2          # tokens not a multiple of 32
    assert pack(qkv.Desc.make(1, 2, 32, 64, 32), [0, 32, 0, 0]) == -2           # head_dim 64 needs a multiple of 64
    assert pack(qkv.Desc.make(1, 1, 16, 256, 32), [0, 16, 0, 0]) == -2          # head_dim 256
    assert pack(qkv.Desc.make(1, 1, 64, 128, 32), [32, 32, 0, 0]) == -7         # not uniform
    assert pack(qkv.Desc.make(1, 1, 64, 128, 32), [0, 0, 0, 64]) == -7          # fp16 rows have no groups
    d = qkv.Desc.make(1, 1, 48, 128, 32)
    assert L.qkv_unpack_dequant_kc(card.data_ptr(), card.numel(), ctypes.byref(d), K.data_ptr(), K.data_ptr(), None, None) == -2
    torch.cuda.synchronize()


def test_random_shapes():
    rng = np.random.default_rng(77)
    for case in range(12):
        D = int(rng.choice([64, 128]))
        step = 64 if D == 64 else 32
        T = step * int(rng.integers(1, 40))
        L = int(rng.integers(1, 5))
        H = int(rng.integers(1, 5))
        width = int(rng.choice([2, 4, 8]))
        run(L, H, T, D, width, 500 + case, "kc random %d: L=%d H=%d T=%d D=%d width=%d" % (case, L, H, T, D, width))


@pytest.mark.parametrize("D,T", [(128, 96), (64, 128)])
@pytest.mark.parametrize("width", [2, 4, 8])
def test_injection_of_per_channel_cards_with_realignment(D, T, width):
    from oracle import inject_ref
    L, H = 4, 2
    say("kc inject D=%d T=%d width=%d" % (D, T, width))
    K, V, bits, counts, desc, rdesc = problem(L, H, T, D, width, 900 + D + width)
    card = torch.empty(qkv.card_bytes(desc, counts), dtype=torch.uint8, device=DEV)
    qkv.quantize_pack_kc(desc, K.to(DEV), V.to(DEV), torch.from_numpy(bits).to(DEV), counts, card)
    torch.cuda.synchronize()
    host = card.cpu().numpy()
    canary, prefix, cap = 0x7E11, 5, T + 9
    for lb, n, rope in ((0, 4, None), (1, 2, (10000.0, 77)), (3, 1, (500000.0, -3)), (0, 4, (10000.0, 4096))):
        kc_ = [torch.zeros((H, cap, D), dtype=torch.int16, device=DEV).fill_(canary).view(torch.float16) for _ in range(n)]
        vc_ = [torch.zeros((H, cap, D), dtype=torch.int16, device=DEV).fill_(canary).view(torch.float16) for _ in range(n)]
        status = torch.ones(1, dtype=torch.int32, device=DEV)
        qkv.inject_layers(card, desc, [k[:, prefix:prefix + T] for k in kc_], [v[:, prefix:prefix + T] for v in vc_], lb,
                          rope_base=rope[0] if rope else 0.0, rope_delta=rope[1] if rope else 0, status=status,
                          keys_per_channel=True)
        torch.cuda.synchronize()
        assert int(status.item()) == 0
        wk = [np.full((H, cap, D), canary, np.uint16) for _ in range(n)]
        wv = [np.full((H, cap, D), canary, np.uint16) for _ in range(n)]
        inject_ref.inject_layers(host, rdesc, wk, wv, lb, prefix, rope, keys_per_channel=True)
        for i in range(n):
            assert np.array_equal(kc_[i].view(torch.int16).cpu().numpy().view(np.uint16), wk[i]), (lb, n, rope, i)
            assert np.array_equal(vc_[i].view(torch.int16).cpu().numpy().view(np.uint16), wv[i]), (lb, n, rope, i)
