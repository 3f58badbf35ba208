"""GPU parity of the controller: network scores and the objective-greedy allocator, through the C ABI,
against the CPU oracle.  Bar: scores bit-identical (both sides run the same fp32 fma chains in the same
order), widths and class counts identical."""
import numpy as np
import pytest
import torch

import paper_2605_03884_amd as qkv
import qkv_synth
from oracle import ref

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print("[case] " + msg, flush=True)


def net(seed):
    w1, b1, w2 = [a.numpy() for a in qkv_synth.make_controller(seed)]
    return w1, b1, w2, qkv.Controller.make(w1, b1, w2)


@pytest.mark.parametrize("T", [1, 63, 64, 257, 1000, 8192, 33333])
def test_scores_match_oracle_bit_for_bit(T):
    say("controller_scores T=%d" % T)
    w1, b1, w2, params = net(100 + T)
    x = qkv_synth.make_features(T, 200 + T).numpy()
    got = qkv.controller_scores(torch.from_numpy(x).to(DEV), params)
    torch.cuda.synchronize()
    want = ref.controller_scores(x, w1, b1, w2)
    assert np.array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32))


def test_scores_special_values():
    say("controller_scores special values")
    rng = np.random.default_rng(7)
    w1 = rng.standard_normal((64, 6)).astype(np.float32)
    b1 = rng.standard_normal(64).astype(np.float32)
    w2 = rng.standard_normal(64).astype(np.float32)          # signed output weights
    b1[3] = np.nan                                           # a NaN pre-activation counts as 0
    w1[9, :] = 0
    b1[9] = -0.0
    x = rng.standard_normal((512, 6)).astype(np.float32)
    x[5] = 0
    x[6] = 1e-39                                             # subnormal features
    x[7] = 3e38
    x[8, 2] = -3e38
    got = qkv.controller_scores(torch.from_numpy(x).to(DEV), qkv.Controller.make(w1, b1, w2))
    torch.cuda.synchronize()
    want = ref.controller_scores(x, w1, b1, w2)
    assert np.array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32))


def test_scores_hand_fixtures_on_the_device():
    # the two rounding fixtures of the oracle's pins, run on the device
    w1 = np.zeros((64, 6), np.float32); b1 = np.zeros(64, np.float32); w2 = np.zeros(64, np.float32)
    a = np.float32(1 + 2.0 ** -12)
    w1[0, 0], b1[0], w2[0] = a, -1, 1
    x = np.zeros((1, 6), np.float32)
    x[0, 0] = a
    got = qkv.controller_scores(torch.from_numpy(x).to(DEV), qkv.Controller.make(w1, b1, w2))
    assert got.item() == 2.0 ** -11 + 2.0 ** -24
    w1[:] = 0
    b1[:3] = [2.0 ** 24, 1, 2.0 ** 24]
    w2[:3] = [1, 1, -1]
    got = qkv.controller_scores(torch.zeros((1, 6), device=DEV), qkv.Controller.make(w1, b1, w2))
    assert got.item() == 0.0


def score_variants(T, rng):
    return {
        "uniform": rng.random(T).astype(np.float32),
        "ties": (np.round(rng.random(T) * 7) / 7).astype(np.float32),
        "all equal": np.full(T, 0.25, dtype=np.float32),
        "signed": rng.standard_normal(T).astype(np.float32),
        "tiny": rng.choice(np.array([0.0, -0.0, 1e-40, 3e-45, 1e-38, np.nan], dtype=np.float32), size=T),
        "sorted": np.sort(rng.random(T).astype(np.float32)),
        "wide": np.exp(rng.standard_normal(T) * 6).astype(np.float32),
        "infs": rng.choice(np.array([np.inf, 0.0, 1.0, 65535.0 / 32], dtype=np.float32), size=T),
    }


@pytest.mark.parametrize("T", [1, 2, 7, 100, 1023, 1024, 1025, 4097, 8192, 8193, 20000, 32768, 32769, 50001])
def test_greedy_matches_oracle(T):
    say("assign_bits_greedy T=%d" % T)
    rng = np.random.default_rng(T)
    for name, scores in score_variants(T, rng).items():
        sd = torch.from_numpy(scores).to(DEV)
        for budget in (2.0, 2.001, 2.5, 3.0, 4.0, 5.0, 7.5, 12.0, 15.999, 16.0):
            bits, counts = qkv.assign_bits_greedy(sd, budget)
            torch.cuda.synchronize()
            wb, wc = ref.assign_bits_greedy(scores, budget)
            got = bits.cpu().numpy()
            assert np.array_equal(got, wb), (name, budget, int(np.flatnonzero(got != wb)[0]))
            assert counts.cpu().tolist() == wc.tolist(), (name, budget)


def test_greedy_without_counts_and_into_given_buffers():
    s = qkv_synth.make_scores(3000, 5, DEV)
    bits = torch.zeros(3000, dtype=torch.uint8, device=DEV)
    rc = qkv.lib().qkv_assign_bits_greedy(s.data_ptr(), 3000, 4.0, bits.data_ptr(), None, None)
    torch.cuda.synchronize()
    assert rc == 0
    assert np.array_equal(bits.cpu().numpy(), ref.assign_bits_greedy(s.cpu().numpy(), 4.0)[0])


def test_features_to_card_chain():
    # features -> scores -> widths -> card, every step on the device, against the same chain in the oracle
    say("controller chain into a card")
    L, H, T, D, G = 2, 2, 1500, 128, 32
    w1, b1, w2, params = net(77)
    x = qkv_synth.make_features(T, 78)
    K, V = qkv_synth.make_kv(L, H, T, D, 79, "llama")
    desc = qkv.Desc.make(L, H, T, D, G, model_id=5, sender_id=6)
    scores = qkv.controller_scores(x.to(DEV), params)
    bits, counts_dev = qkv.assign_bits_greedy(scores, 3.5)
    counts = counts_dev.cpu().tolist()
    card = torch.empty(qkv.card_bytes(desc, counts), dtype=torch.uint8, device=DEV)
    qkv.quantize_pack(desc, K.to(DEV), V.to(DEV), bits, counts, card)
    torch.cuda.synchronize()
    ws = ref.controller_scores(x.numpy(), w1, b1, w2)
    wb, wc = ref.assign_bits_greedy(ws, 3.5)
    assert counts == wc.tolist() and len(set(wb.tolist())) >= 2
    want = ref.quantize_pack(ref.make_desc(L, H, T, D, G, 5, 6, 0), K.numpy().view(np.uint16), V.numpy().view(np.uint16),
                             wb, wc)
    assert np.array_equal(card.cpu().numpy(), want)


def test_controller_errors():
    s = torch.zeros(16, dtype=torch.float32, device=DEV)
    f = torch.zeros((16, 6), dtype=torch.float32, device=DEV)
    b = torch.zeros(16, dtype=torch.uint8, device=DEV)
    L = qkv.lib()
    p = qkv.Controller()
    import ctypes
    assert L.qkv_controller_scores(None, 16, ctypes.byref(p), s.data_ptr(), None) == -1
    assert L.qkv_controller_scores(f.data_ptr(), 16, None, s.data_ptr(), None) == -1
    assert L.qkv_controller_scores(f.data_ptr(), 0, ctypes.byref(p), s.data_ptr(), None) == -2
    assert L.qkv_controller_scores(f.data_ptr() + 4, 8, ctypes.byref(p), s.data_ptr(), None) == -6
    assert L.qkv_assign_bits_greedy(None, 16, 4.0, b.data_ptr(), None, None) == -1
    assert L.qkv_assign_bits_greedy(s.data_ptr(), 0, 4.0, b.data_ptr(), None, None) == -2
    assert L.qkv_assign_bits_greedy(s.data_ptr(), 1 << 28, 4.0, b.data_ptr(), None, None) == -2
    for bad in (1.99, 16.01, float("nan")):
        assert L.qkv_assign_bits_greedy(s.data_ptr(), 16, bad, b.data_ptr(), None, None) == -4
    assert L.qkv_assign_bits_greedy(s.data_ptr(), 16, 4.0, b.data_ptr(), s.data_ptr() + 4, None) == -6
    torch.cuda.synchronize()
