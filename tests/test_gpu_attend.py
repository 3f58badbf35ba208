"""GPU parity of the fused attention over a card (qkv_card_attend) against its float64 oracle.

Tolerance (derived from the arithmetic, computed per case from the data): the kernel forms each
score from exact fp16 x fp16 products accumulated in fp32 (at most 128 roundings of relative size
2^-24 on partial sums bounded by sum_i |q_i k_i|), evaluates 2^x with the hardware instruction
(about 1 ulp) and accumulates p.V^ over T tokens in fp32.  So
    |ds|  <= 128 * 2^-24 * scale * max_t sum_i |q_i K^_ti|
    |do|  <= (2 |ds| + (T + 8) * 2^-24 + 2^-21) * max |V^|         (weights sum to one)
    |dlse| <= |ds| + (T + 8) * 2^-24 + 2^-21
These are worst-case bounds; rounding errors do not line up like that, and the observed errors
(printed) are about 1e-6 of max |V^|.  A second, empirical guard of 1e-5 * max(1, max |V^|) for the output
(ten times the largest error seen over all cases) and 1e-4 for the log-sum (five times) is asserted as
well, so that a regression far inside the worst-case bound - a lost tail of small weights, say - is caught.
"""
import math

import numpy as np
import pytest
import torch

import paper_2605_03884_amd as qkv
import qkv_synth
from oracle import attend_ref, ref

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print("[case] " + msg, flush=True)


def build_card(L, H, T, D, G, bits, seed, kind="llama"):
    K, V = qkv_synth.make_kv(L, H, T, D, seed, kind)
    counts = [int((bits == w).sum()) for w in (2, 4, 8, 16)]
    rd = ref.make_desc(L, H, T, D, G)
    card = ref.quantize_pack(rd, K.numpy(), V.numpy(), bits, counts)     # the oracle's card: the attention kernel is what is under test
    return rd, card


def run_gpu(card, L, H, T, D, G, q, scale, with_lse=True):
    desc = qkv.Desc.make(L, H, T, D, G)
    card_dev = torch.from_numpy(card).to(DEV)
    q_dev = torch.from_numpy(q).to(DEV)
    out = torch.full((L, q.shape[1], D), float("nan"), dtype=torch.float32, device=DEV)
    lse = torch.full((L, q.shape[1]), float("nan"), dtype=torch.float32, device=DEV) if with_lse else None
    status = torch.full((1,), 0x7777, dtype=torch.int32, device=DEV)
    qkv.card_attend(card_dev, desc, q_dev, scale, out, lse=lse, status=status)
    torch.cuda.synchronize()
    return out.cpu().numpy(), (lse.cpu().numpy() if with_lse else None), int(status.item())


def bounds(card, rd, q, scale):
    kq, vq = ref.unpack_dequant(card, rd)
    Kf = np.abs(kq.view(np.float16).astype(np.float64))
    rep = q.shape[1] // rd.kv_heads
    ds = 0.0
    for l in range(rd.layers):
        for hq in range(q.shape[1]):
            ds = max(ds, float((Kf[l, hq // rep] @ np.abs(q[l, hq].astype(np.float64))).max()))
    ds *= rd.head_dim * 2.0 ** -24 * scale
    vmax = float(np.abs(vq.view(np.float16).astype(np.float64)).max())
    base = (rd.tokens + 8) * 2.0 ** -24 + 2.0 ** -21
    return min((2 * ds + base) * vmax, 1e-5 * max(1.0, vmax)), min(ds + base, 1e-4)


def check(L, H, rep, T, G, bits, seed, label, scale=None, kind="llama", D=128):
    say(label)
    scale = D ** -0.5 if scale is None else scale
    rd, card = build_card(L, H, T, D, G, bits, seed, kind)
    q = np.random.default_rng(seed + 1).standard_normal((L, H * rep, D)).astype(np.float16)
    out, lse, st = run_gpu(card, L, H, T, D, G, q, scale)
    assert st == 0
    want_o, want_lse = attend_ref.card_attend(card, rd, q, scale)
    tol_o, tol_lse = bounds(card, rd, q, scale)
    err_o = float(np.abs(out - want_o).max())
    err_l = float(np.abs(lse - want_lse).max())
    print("        max |do| %.3g (bound %.3g)   max |dlse| %.3g (bound %.3g)" % (err_o, tol_o, err_l, tol_lse), flush=True)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    assert err_o <= tol_o and err_l <= tol_lse
    return err_o, tol_o


@pytest.mark.parametrize("T", [1, 15, 16, 17, 100, 511, 512, 513, 1500])
def test_token_counts_around_round_and_task_edges(T):
    bits = qkv_synth.make_bits_uniform_choice(T, 40 + T).numpy()
    check(2, 2, 4, T, 32, bits, 400 + T, "attend T=%d mixed" % T)


@pytest.mark.parametrize("width", [2, 4, 8, 16])
@pytest.mark.parametrize("G", [32, 64, 128])
def test_uniform_cards_every_group_size(width, G):
    T = 700
    check(1, 3, 4, T, G, np.full(T, width, dtype=np.uint8), 500 + width + G, "attend uniform %d-bit G%d" % (width, G))


@pytest.mark.parametrize("rep", [1, 2, 3, 4, 5, 8, 12, 16])
def test_query_heads_per_kv_head(rep):
    T = 900
    bits = qkv_synth.make_bits_uniform_choice(T, 60 + rep).numpy()
    check(2, 2, rep, T, 32, bits, 600 + rep, "attend rep=%d" % rep)


@pytest.mark.parametrize("D,G", [(64, 32), (64, 64), (256, 32), (256, 64), (256, 128)])
@pytest.mark.parametrize("rep", [1, 4, 7, 16])
def test_other_head_dims(D, G, rep):
    """head_dim 64 (half of the kernel's lanes idle) and 256 (two halves of 128), mixed widths, both MFMA forms."""
    T = 600
    bits = qkv_synth.make_bits_uniform_choice(T, 90 + D + rep).numpy()
    check(2, 2, rep, T, G, bits, 900 + D + G + rep, "attend head_dim=%d G=%d rep=%d" % (D, G, rep), D=D)


@pytest.mark.parametrize("D", [64, 256])
@pytest.mark.parametrize("width", [2, 4, 8, 16])
def test_other_head_dims_uniform_widths_and_ragged_tasks(D, width):
    for T in (1, 17, 385, 1000):
        check(1, 2, 4, T, 32, np.full(T, width, dtype=np.uint8), 950 + D + width + T,
              "attend head_dim=%d uniform %d-bit T=%d" % (D, width, T), D=D)


def check_kc(L, H, rep, T, D, width, seed, label, kind="llama"):
    """Attention over a uniform card whose keys are grouped per channel, against the same float64 definition."""
    say(label)
    G, scale = 32, D ** -0.5
    K, V = qkv_synth.make_kv(L, H, T, D, seed, kind)
    bits = np.full(T, width, dtype=np.uint8)
    counts = [T if width == w else 0 for w in (2, 4, 8, 16)]
    rd = ref.make_desc(L, H, T, D, G)
    card = ref.quantize_pack_kc(rd, K.numpy(), V.numpy(), bits, counts)
    q = np.random.default_rng(seed + 1).standard_normal((L, H * rep, D)).astype(np.float16)
    desc = qkv.Desc.make(L, H, T, D, G)
    card_dev = torch.from_numpy(card).to(DEV)
    out = torch.full((L, H * rep, D), float("nan"), dtype=torch.float32, device=DEV)
    lse = torch.full((L, H * rep), float("nan"), dtype=torch.float32, device=DEV)
    status = torch.full((1,), 0x7777, dtype=torch.int32, device=DEV)
    qkv.card_attend_kc(card_dev, desc, torch.from_numpy(q).to(DEV), scale, out, lse=lse, status=status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    want_o, want_lse = attend_ref.card_attend(card, rd, q, scale, keys_per_channel=True)
    kq, vq = ref.unpack_dequant_kc(card, rd)
    Kf = np.abs(kq.view(np.float16).astype(np.float64))
    ds = max(float((Kf[l, hq // rep] @ np.abs(q[l, hq].astype(np.float64))).max()) for l in range(L) for hq in range(H * rep))
    ds *= D * 2.0 ** -24 * scale
    vmax = float(np.abs(vq.view(np.float16).astype(np.float64)).max())
    base = (T + 8) * 2.0 ** -24 + 2.0 ** -21
    tol_o, tol_lse = min((2 * ds + base) * vmax, 1e-5 * max(1.0, vmax)), min(ds + base, 1e-4)
    err_o, err_l = float(np.abs(out.cpu().numpy() - want_o).max()), float(np.abs(lse.cpu().numpy() - want_lse).max())
    print("        max |do| %.3g (bound %.3g)   max |dlse| %.3g (bound %.3g)" % (err_o, tol_o, err_l, tol_lse), flush=True)
    assert err_o <= tol_o and err_l <= tol_lse
    return card_dev, desc, q


@pytest.mark.parametrize("width", [2, 4, 8])
@pytest.mark.parametrize("D,T", [(128, 32), (128, 96), (128, 128), (128, 320), (128, 416), (128, 1024), (64, 64), (64, 320), (64, 448),
                                 (64, 1024)])
def test_cards_grouped_per_channel(width, D, T):
    """Token counts below, at and across the 128-token super-blocks and the 384-token tasks; tasks of exactly 128 tokens,
    where the softmax's granularity at 4 bits (48 tokens) reaches past the last super-block that holds a token."""
    check_kc(2, 2, 4, T, D, width, 1100 + width + D + T, "attend per-channel keys head_dim=%d %d-bit T=%d" % (D, width, T))


@pytest.mark.parametrize("rep", [1, 3, 8, 16])
def test_cards_grouped_per_channel_query_head_counts(rep):
    check_kc(1, 2, rep, 800, 128, 4, 1200 + rep, "attend per-channel keys rep=%d" % rep)
    check_kc(1, 2, rep, 768, 64, 2, 1300 + rep, "attend per-channel keys head_dim=64 rep=%d" % rep)
    check_kc(3, 4, rep, 320, 64, 4, 1350 + rep, "attend per-channel keys head_dim=64 4-bit T=320 rep=%d" % rep)


def test_cards_grouped_per_channel_are_told_apart():
    """Each of the two calls refuses a card of the other grouping on the device and leaves the outputs alone."""
    card_dev, desc, q = check_kc(1, 2, 4, 256, 128, 4, 1400, "attend per-channel keys, then the wrong call")
    out = torch.full((1, 8, 128), float("nan"), dtype=torch.float32, device=DEV)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    qkv.card_attend(card_dev, desc, torch.from_numpy(q).to(DEV), 1.0, out, status=status)
    torch.cuda.synchronize()
    assert int(status.item()) == qkv.STATUS_BAD_HEADER and bool(torch.isnan(out).all())
    rd, card = build_card(1, 2, 256, 128, 32, np.full(256, 4, dtype=np.uint8), 1401)
    qkv.card_attend_kc(torch.from_numpy(card).to(DEV), desc, torch.from_numpy(q).to(DEV), 1.0, out, status=status)
    torch.cuda.synchronize()
    assert int(status.item()) == qkv.STATUS_BAD_HEADER and bool(torch.isnan(out).all())
    with pytest.raises(qkv.QkvError) as e:       # group size 64 has no per-channel form
        qkv.card_attend_kc(card_dev, qkv.Desc.make(1, 2, 256, 128, 64), torch.from_numpy(q).to(DEV), 1.0, out)
    assert e.value.code == -3
    with pytest.raises(qkv.QkvError) as e:       # tokens not a multiple of 32
        qkv.card_attend_kc(card_dev, qkv.Desc.make(1, 2, 250, 128, 32), torch.from_numpy(q).to(DEV), 1.0, out)
    assert e.value.code == -2


def test_skewed_mixes_empty_classes_and_scales():
    T = 1100
    rng = np.random.default_rng(8)
    for probs in [(0.97, 0.01, 0.01, 0.01), (0.0, 0.5, 0.0, 0.5), (0.0, 0.0, 0.0, 1.0), (0.5, 0.0, 0.5, 0.0)]:
        bits = rng.choice(np.array([2, 4, 8, 16], dtype=np.uint8), size=T, p=probs)
        check(1, 2, 4, T, 32, bits, 700, "attend mix %r" % (probs,))
    bits = qkv_synth.make_bits_uniform_choice(T, 71).numpy()
    check(1, 2, 4, T, 32, bits, 701, "attend scale 1.0 (peaked softmax)", scale=1.0)
    check(1, 2, 4, T, 32, bits, 702, "attend scale 0 (uniform weights)", scale=0.0)


def test_many_tiny_weights_still_count():
    # one dominant token and thousands of tokens whose weights span 1e-4 .. 1e-11 but whose values are
    # large: the small weights must not be lost (they pass through fp16 operands inside the kernel)
    L, H, rep, T, D, G = 1, 1, 4, 4096, 128, 32
    rng = np.random.default_rng(12)
    K = np.zeros((L, H, T, D), dtype=np.float16)
    V = (rng.standard_normal((L, H, T, D)) * 500).astype(np.float16)
    K[0, 0, 1:, 0] = -rng.uniform(9.0, 25.0, size=T - 1).astype(np.float16)      # scores -9 .. -25 against token 0's 0
    V[0, 0, 0] = 1.0
    q = np.zeros((L, H * rep, D), dtype=np.float16)
    q[:, :, 0] = 1.0
    bits = np.full(T, 16, dtype=np.uint8)                                        # raw rows: K^ = K exactly
    rd = ref.make_desc(L, H, T, D, G)
    card = ref.quantize_pack(rd, K, V, bits, [0, 0, 0, T])
    say("attend: many tiny weights")
    out, lse, st = run_gpu(card, L, H, T, D, G, q, 1.0)
    want_o, want_lse = attend_ref.card_attend(card, rd, q, 1.0)
    assert st == 0
    # the tail carries a visible share of the result
    assert np.abs(want_o[0, 0] - 1.0).max() > 1e-2
    err = float(np.abs(out - want_o).max())
    print("        max |do| %.3g, |o| up to %.3g" % (err, float(np.abs(want_o).max())), flush=True)
    assert err <= 2e-5 * float(np.abs(want_o).max()) + 1e-6
    assert np.abs(lse - want_lse).max() <= 1e-5


def test_matches_attention_over_the_gpu_dequantized_cache():
    # same numbers as running the injection kernel first and attending over the dense cache
    L, H, rep, T, D, G = 2, 2, 4, 640, 128, 32
    bits = qkv_synth.make_bits_uniform_choice(T, 81).numpy()
    rd, card = build_card(L, H, T, D, G, bits, 800)
    desc = qkv.Desc.make(L, H, T, D, G)
    card_dev = torch.from_numpy(card).to(DEV)
    K = torch.empty((L, H, T, D), dtype=torch.float16, device=DEV)
    V = torch.empty_like(K)
    qkv.unpack_dequant(card_dev, desc, K, V)
    q = np.random.default_rng(3).standard_normal((L, H * rep, D)).astype(np.float16)
    out, lse, st = run_gpu(card, L, H, T, D, G, q, D ** -0.5)
    o2, l2 = attend_ref.attend_dense(q, K.cpu().numpy(), V.cpu().numpy(), D ** -0.5)
    tol_o, tol_l = bounds(card, rd, q, D ** -0.5)
    assert np.abs(out - o2).max() <= tol_o and np.abs(lse - l2).max() <= tol_l


def test_bad_header_leaves_outputs_untouched_and_errors_are_reported():
    L, H, rep, T, D, G = 1, 2, 4, 200, 128, 32
    bits = qkv_synth.make_bits_uniform_choice(T, 91).numpy()
    rd, card = build_card(L, H, T, D, G, bits, 900)
    q = np.zeros((L, H * rep, D), dtype=np.float16)
    bad = card.copy()
    bad[0] = ord("X")
    out, lse, st = run_gpu(bad, L, H, T, D, G, q, 1.0)
    assert st == qkv.STATUS_BAD_HEADER and np.isnan(out).all() and np.isnan(lse).all()
    out, lse, st = run_gpu(card, L, H, T, D, G, q, 1.0, with_lse=False)
    assert st == 0 and np.isfinite(out).all()
    desc = qkv.Desc.make(L, H, T, D, G)
    card_dev = torch.from_numpy(card).to(DEV)
    q_dev = torch.from_numpy(q).to(DEV)
    o = torch.empty((L, H * rep, D), dtype=torch.float32, device=DEV)
    with pytest.raises(qkv.QkvError) as e:       # workspace too small
        qkv.card_attend(card_dev, desc, q_dev, 1.0, o, workspace=torch.empty(64, dtype=torch.uint8, device=DEV))
    assert e.value.code == -5
    with pytest.raises(qkv.QkvError) as e:       # 17 query heads per kv head
        qkv.card_attend_workspace(desc, 34)
    assert e.value.code == -2
    with pytest.raises(qkv.QkvError) as e:       # a head_dim no card can have
        qkv.card_attend_workspace(qkv.Desc.make(L, H, T, 96, 32), 8)
    assert e.value.code == -2
    # a card of another head_dim than the caller expects is refused on the device, like any foreign header
    q256 = np.zeros((L, H * rep, 256), dtype=np.float16)
    out, lse, st = run_gpu(card, L, H, T, 256, G, q256, 1.0)
    assert st == qkv.STATUS_BAD_HEADER and np.isnan(out).all() and np.isnan(lse).all()


def test_benchmark_shape_8k():
    cfg = qkv_synth.CONFIGS["llama8b_8k_b3"]
    L, H, T, D, G = cfg["layers"], cfg["kv_heads"], cfg["tokens"], cfg["head_dim"], cfg["group_size"]
    say("attend 8K: building the card on the GPU")
    K, V = qkv_synth.make_kv(L, H, T, D, cfg["data_seed"], cfg["kind"], device=DEV)
    scores = qkv_synth.make_scores(T, cfg["bits"][1], DEV)
    bits, counts = qkv.assign_bits(scores, cfg["bits"][2])
    desc = qkv.Desc.make(L, H, T, D, G)
    card_dev = torch.empty(qkv.card_bytes(desc, counts), dtype=torch.uint8, device=DEV)
    qkv.quantize_pack(desc, K, V, bits, counts, card_dev)
    rep = 4
    q = np.random.default_rng(5).standard_normal((L, H * rep, D)).astype(np.float16)
    out = torch.empty((L, H * rep, D), dtype=torch.float32, device=DEV)
    lse = torch.empty((L, H * rep), dtype=torch.float32, device=DEV)
    status = torch.ones(1, dtype=torch.int32, device=DEV)
    qkv.card_attend(card_dev, desc, torch.from_numpy(q).to(DEV), D ** -0.5, out, lse=lse, status=status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    say("attend 8K: oracle")
    rd = ref.make_desc(L, H, T, D, G)
    # the oracle's own card from the same seeded inputs (never the GPU's)
    want_bits, want_counts = ref.assign_bits(qkv_synth.make_scores(T, cfg["bits"][1]).numpy(), cfg["bits"][2])
    card = ref.quantize_pack(rd, K.cpu().numpy(), V.cpu().numpy(), want_bits, want_counts)
    want_o, want_lse = attend_ref.card_attend(card, rd, q, D ** -0.5)
    tol_o, tol_l = bounds(card, rd, q, D ** -0.5)
    err_o = float(np.abs(out.cpu().numpy() - want_o).max())
    err_l = float(np.abs(lse.cpu().numpy() - want_lse).max())
    print("        max |do| %.3g (bound %.3g)   max |dlse| %.3g (bound %.3g)" % (err_o, tol_o, err_l, tol_l), flush=True)
    assert err_o <= tol_o and err_l <= tol_l


def test_several_query_tokens_in_one_pass():
    """Three new tokens x four query heads per kv head as twelve "heads": one pass over the card, each token's
    slice against the oracle."""
    L, H, R, S, T, D, G = 2, 2, 4, 3, 900, 128, 32
    say("attend: %d query tokens in one pass" % S)
    K, V = qkv_synth.make_kv(L, H, T, D, 801, "llama")
    bits = qkv_synth.make_bits_uniform_choice(T, 802).numpy()
    counts = ref.count_bits(bits).tolist()
    rd = ref.make_desc(L, H, T, D, G)
    card = ref.quantize_pack(rd, K.numpy().view(np.uint16), V.numpy().view(np.uint16), bits, counts)
    desc = qkv.Desc.make(L, H, T, D, G)
    q_tok = np.random.default_rng(803).standard_normal((S, L, H * R, D)).astype(np.float16)      # per token [L][Hq][D]
    # [S][L][H][R][D] -> [L][H][S][R][D]
    q_all = np.ascontiguousarray(q_tok.reshape(S, L, H, R, D).transpose(1, 2, 0, 3, 4)).reshape(L, H * S * R, D)
    out = torch.empty((L, H * S * R, D), dtype=torch.float32, device=DEV)
    lse = torch.empty((L, H * S * R), dtype=torch.float32, device=DEV)
    status = torch.ones(1, dtype=torch.int32, device=DEV)
    qkv.card_attend(torch.from_numpy(card).to(DEV), desc, torch.from_numpy(q_all).to(DEV), D ** -0.5, out, lse=lse, status=status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    got_o = out.cpu().numpy().reshape(L, H, S, R, D)
    got_l = lse.cpu().numpy().reshape(L, H, S, R)
    for s_ in range(S):
        want_o, want_l = attend_ref.card_attend(card, rd, q_tok[s_], D ** -0.5)
        tol_o, tol_l = bounds(card, rd, q_tok[s_], D ** -0.5)
        assert np.abs(got_o[:, :, s_].reshape(L, H * R, D) - want_o).max() <= tol_o
        assert np.abs(got_l[:, :, s_].reshape(L, H * R) - want_l).max() <= tol_l
