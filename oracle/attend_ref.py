"""CPU oracle for decode-step attention over a CacheCard (paper Sec. 4.3: consuming a
foreign quantized cache directly inside attention, which the paper leaves as future work).

TEST INFRASTRUCTURE ONLY, like the rest of oracle/.  The result has a plain definition, so
the oracle is that definition written out in float64: the card is first dequantized to the
dense fp16 cache exactly as the receiver-side injection would produce it (oracle/ref.py,
Sec. 4.2.2), then for every layer l and query head hq, with kv head h = hq // (Hq / H):

    s_t   = scale * <q[l, hq], K^[l, h, t]>          t = 0 .. T-1
    lse   = log sum_t exp(s_t)
    o     = sum_t exp(s_t - lse) * V^[l, h, t]

There is no blocking, no running maximum carried between blocks and no reordering; the
maximum is subtracted once, as the textbook softmax does, to keep exp() in range.

Pins (tests marked "not gpu"): one token; zero query (o = mean of V^); identical keys;
a dominant key; invariance under a permutation of the tokens; the two-token closed form with
the logistic function; the merge identity of two disjoint token sets; pure-Python loops on
tiny inputs.
"""
import numpy as np

from . import ref


def attend_dense(q, K, V, scale):
    """q: [L, Hq, D]; K, V: [L, H, T, D] (any float dtype).  Returns (o [L, Hq, D], lse [L, Hq]) in float64."""
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    L, Hq, D = q.shape
    H = K.shape[1]
    assert K.shape == V.shape and K.shape[0] == L and K.shape[3] == D and Hq % H == 0
    rep = Hq // H
    o = np.zeros((L, Hq, D), dtype=np.float64)
    lse = np.zeros((L, Hq), dtype=np.float64)
    for l in range(L):
        for hq in range(Hq):
            h = hq // rep
            s = scale * (K[l, h] @ q[l, hq])              # [T]
            m = s.max()
            p = np.exp(s - m)
            z = p.sum()
            lse[l, hq] = m + np.log(z)
            o[l, hq] = (p[:, None] * V[l, h]).sum(axis=0) / z
    return o, lse


def card_attend(card, desc, q, scale, keys_per_channel=False):
    """card: uint8 array; desc: ref.RefDesc of the card; q: float16 [L, Hq, D].  keys_per_channel: the card is a
    uniform card whose key groups run along the tokens of one channel (Sec. 2's per-channel key scheme); the
    definition is the same, over the cache that card dequantizes to."""
    k_bits, v_bits = (ref.unpack_dequant_kc if keys_per_channel else ref.unpack_dequant)(card, desc)
    return attend_dense(q, k_bits.view(np.float16), v_bits.view(np.float16), scale)
