"""Random shapes, width mixes and planted special values, each taken through every call on the same card: card
creation and injection against the oracle byte for byte, a layer range into per-layer caches with or without key
realignment, one hop card to card at other widths, attention over the card, and the per-channel-key calls where
the shape allows them.  The checks are the ones of the per-call test files (imported from there); this file adds
the chaining, other seeds, and value patterns planted into random groups."""
import numpy as np
import pytest
import torch

import paper_2605_03884_amd as qkv
from oracle import attend_ref, ref

import test_gpu_attend as att
import test_gpu_inject as inj
import test_gpu_kc as kc
import test_gpu_parity as par
import test_gpu_requant as rq

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def plant(x, rng):
    """A few groups of 32 values replaced by: a constant, signed zeros, subnormals, values near the fp16 maximum,
    neighbouring fp16 numbers, a tiny range."""
    flat = x.reshape(-1, 32)
    for _ in range(int(rng.integers(0, 6))):
        g = int(rng.integers(0, flat.shape[0]))
        kind = int(rng.integers(0, 6))
        if kind == 0:
            flat[g] = np.float16(rng.standard_normal())
        elif kind == 1:
            flat[g] = np.where(rng.random(32) < 0.5, np.float16(0.0), np.float16(-0.0))
        elif kind == 2:
            flat[g] = rng.integers(0, 1024, 32).astype(np.uint16).view(np.float16)
        elif kind == 3:
            flat[g] = np.float16(60000.0) * np.sign(rng.standard_normal(32)).astype(np.float16)
        elif kind == 4:
            flat[g] = (rng.integers(0, 3, 32).astype(np.uint16) + np.uint16(0x3C00)).view(np.float16)
        else:
            flat[g] = (rng.standard_normal(32) * 1e-6).astype(np.float16)
    return x


def rigorous_bounds(card, rd, q, scale, lse):
    """The error bounds of fp32 accumulation without the per-call tests' empirical cap: planted values near the fp16
    maximum make sum |q_i K^_i| huge, and then the honest bound is what holds.  |ds| <= head_dim * 2^-24 * scale * max sum |q K^|;
    |d lse| <= |ds| + (T + 8) * 2^-24 + 2^-21 + a few fp32 roundings of lse itself; |d out| <= (2 |ds| + ...) * max |V^|."""
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
    return (2 * ds + base) * max(vmax, 1e-30), ds + base + 4e-6 * max(1.0, float(np.abs(lse).max()))


@pytest.mark.parametrize("seed", [101, 202, 303, 404])
def test_every_call_on_random_cards(seed):
    rng = np.random.default_rng(seed)
    for case in range(12):
        D = int(rng.choice([64, 128, 128, 128, 256]))
        G = int(rng.choice([g for g in (32, 64, 128) if g <= D]))
        L, H = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        T = int(rng.choice([rng.integers(1, 40), rng.integers(1, 700), rng.integers(700, 2000)]))
        probs = rng.dirichlet(np.ones(4) * float(rng.choice([0.2, 0.6, 3.0])))
        bits = rng.choice(np.array([2, 4, 8, 16], dtype=np.uint8), size=T, p=probs)
        kind = "llama" if rng.random() < 0.5 else "tiny"
        s = int(rng.integers(1, 1 << 30))
        label = "seed %d case %d: L%d H%d T%d D%d G%d %s" % (seed, case, L, H, T, D, G, kind)
        desc, K, V = par.make_problem(L, H, T, D, G, seed=s, kind=kind)
        K, V = plant(K.copy(), rng), plant(V.copy(), rng)
        card, _, _ = par.check_round_trip(desc, K, V, bits, label)
        rdesc = par.ref_desc(desc)
        card_dev = torch.from_numpy(card).to(DEV)

        lb = int(rng.integers(0, L))
        count = int(rng.integers(1, L - lb + 1))
        prefix = int(rng.integers(0, 9))
        cap = T + prefix + int(rng.integers(0, 5))
        rope = None if rng.random() < 0.4 else (float(rng.choice([10000.0, 500000.0])), int(rng.integers(-5000, 200000)))
        inj.check(desc, rdesc, card_dev, card, lb, count, cap, prefix, rope, label + ", injection")

        bits2 = rng.choice(np.array([2, 4, 8, 16], dtype=np.uint8), size=T, p=rng.dirichlet(np.ones(4) * 0.6))
        counts2 = ref.count_bits(bits2).tolist()
        rd2 = ref.make_desc(L, H, T, D, G, 7, 8, 9)
        want = rq.oracle_hop(card, rdesc, rd2, bits2, counts2)
        desc2 = qkv.Desc.make(L, H, T, D, G, model_id=7, sender_id=8, position_offset=9)
        out = torch.full((want.size + 256,), 0xA5, dtype=torch.uint8, device=DEV)
        status = torch.full((1,), 0x7777, dtype=torch.int32, device=DEV)
        qkv.requantize(card_dev, desc2, torch.from_numpy(bits2).to(DEV), counts2, out[:want.size], status=status)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert int(status.item()) == 0 and np.all(got[want.size:] == 0xA5), label
        assert np.array_equal(got[:want.size], want), label + ", requantized card differs"

        if True:                                             # every head_dim the card format has
            rep = int(rng.choice([1, 2, 4, 8, 16]))
            q = (rng.standard_normal((L, H * rep, D)) * float(rng.choice([0.3, 1.0, 3.0]))).astype(np.float16)
            scale = float(rng.choice([D ** -0.5, 0.02, 0.3]))
            go, gl, st = att.run_gpu(card, L, H, T, D, G, q, scale)
            wo, wl = attend_ref.card_attend(card, rdesc, q, scale)
            assert st == 0
            if np.isfinite(wo).all() and np.isfinite(wl).all():
                tol_o, tol_l = rigorous_bounds(card, rdesc, q, scale, wl)
                assert float(np.abs(go - wo).max()) <= tol_o and float(np.abs(gl - wl).max()) <= tol_l, label + ", attention"

        if G == 32 and D in (64, 128) and T % (64 if D == 64 else 32) == 0:
            width = int(rng.choice([2, 4, 8]))
            kc.run(L, H, T, D, width, s % 100000, label + ", per-channel keys")
            att.check_kc(L, H, int(rng.choice([1, 2, 4, 8, 16])), T, D, width, s % 100000, label + ", attention over per-channel keys", kind=kind)
