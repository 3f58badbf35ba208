"""Pins for the oracle's number handling: fp16 conversion, one-group quantizer, packing.

None of these compares the oracle with itself: each checks it against numpy's IEEE
arithmetic, exact rational arithmetic, a closed form or a hand-written fixture.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import ref

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def f16(bits):
    return np.array(bits, dtype=np.uint16).view(np.float16)


def order_key(h):
    h = np.asarray(h, dtype=np.uint16).astype(np.int64)
    return np.where(h & 0x8000, 0xFFFF - h, h | 0x8000)


# ----------------------------------------------------------------------------- fp16


def test_half_to_float_exhaustive_against_numpy():
    allh = np.arange(65536, dtype=np.uint16)
    want = allh.view(np.float16).astype(np.float32).view(np.uint32)
    got = np.array([np.float32(ref.half_to_float(int(h))).view(np.uint32) for h in allh], dtype=np.uint32)
    nan = (allh & 0x7C00 == 0x7C00) & (allh & 0x3FF != 0)
    assert np.array_equal(got[~nan], want[~nan])
    # NaNs: still NaN, sign and payload carried over (the quiet bit aside: passing a float
    # through the C return value may set it)
    assert np.all((got[nan] & 0x7F800000) == 0x7F800000)
    assert np.all(got[nan] & 0x007FFFFF != 0)
    assert np.array_equal(got[nan] >> 31, allh[nan] >> 15)
    assert np.array_equal((got[nan] >> 13) & 0x1FF, allh[nan] & 0x1FF)


def test_float_to_half_rne_against_numpy():
    # every finite half, the midpoints between neighbours, and one float32 step either side of both
    h = np.arange(0x7C00, dtype=np.uint16)
    v = h.view(np.float16).astype(np.float64)
    mids = (v[:-1] + v[1:]) / 2
    pts = np.concatenate([v, mids, [65504.0, 65519.99, 65520.0, 65536.0, 1e-9, 2.0 ** -25, 2.0 ** -26]]).astype(np.float32)
    cand = np.concatenate([pts, np.nextafter(pts, np.float32(np.inf)), np.nextafter(pts, np.float32(-np.inf))])
    cand = np.concatenate([cand, -cand])
    rng = np.random.default_rng(5)
    rnd = rng.integers(0, 2 ** 32, size=60000, dtype=np.uint64).astype(np.uint32).view(np.float32)
    rnd = rnd[np.isfinite(rnd)]
    cand = np.concatenate([cand, rnd]).astype(np.float32)
    with np.errstate(over="ignore"):
        want = cand.astype(np.float16).view(np.uint16)
    got = np.array([ref.float_to_half(float(x)) for x in cand], dtype=np.uint16)
    assert np.array_equal(got, want)


def test_float_to_half_specials():
    assert ref.float_to_half(float("inf")) == 0x7C00
    assert ref.float_to_half(float("-inf")) == 0xFC00
    assert ref.float_to_half(-0.0) == 0x8000
    n = ref.float_to_half(float("nan"))
    assert (n & 0x7C00) == 0x7C00 and (n & 0x3FF) != 0


# ----------------------------------------------------------------------------- packing


def _golden_pack_rows():
    rows = []
    with open(os.path.join(GOLDEN, "pack_bytes.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w, codes, packed = [s.strip() for s in line.split("|")]
            rows.append((int(w), [int(c) for c in codes.split()], [int(b, 16) for b in packed.split()]))
    return rows


@pytest.mark.parametrize("width,codes,packed", _golden_pack_rows())
def test_pack_bytes_match_hand_computed(width, codes, packed):
    got = ref.pack_codes(np.array(codes, dtype=np.uint8), width)
    assert got.tolist() == packed
    assert ref.unpack_codes(np.array(packed, dtype=np.uint8), len(codes), width).tolist() == codes


@pytest.mark.parametrize("width", [2, 4, 8])
def test_pack_every_pattern_at_every_position(width):
    per_byte = 8 // width
    n = 16
    for pos in range(n):
        for val in range(1 << width):
            codes = np.zeros(n, dtype=np.uint8)
            codes[pos] = val
            packed = ref.pack_codes(codes, width)
            want = np.zeros(n * width // 8, dtype=np.uint8)
            want[pos // per_byte] = val << ((pos % per_byte) * width)
            assert np.array_equal(packed, want)
            assert np.array_equal(ref.unpack_codes(packed, n, width), codes)


@pytest.mark.parametrize("width", [2, 4, 8])
def test_pack_matches_numpy_bit_arithmetic(width):
    rng = np.random.default_rng(width)
    codes = rng.integers(0, 1 << width, size=256, dtype=np.uint8)
    # independent formulation: the row as one little-endian big integer
    big = 0
    for i, c in enumerate(codes.tolist()):
        big |= c << (i * width)
    want = np.frombuffer(big.to_bytes(256 * width // 8, "little"), dtype=np.uint8)
    assert np.array_equal(ref.pack_codes(codes, width), want)


# ----------------------------------------------------------------------------- quantizer


def numpy_quantize(x16, width):
    """Textbook per-group asymmetric min-max quantization in numpy IEEE arithmetic."""
    qmax = (1 << width) - 1
    keys = order_key(x16.view(np.uint16))
    mn = x16[np.argmin(keys)]
    mx = x16[np.argmax(keys)]
    rng_ = np.float32(mx) - np.float32(mn)
    s32 = np.float32(rng_ / np.float32(qmax))
    sh = np.float16(s32)
    s = np.float32(sh)
    inv = np.float32(1.0) / s if s > 0 else np.float32(0.0)
    d = x16.astype(np.float32) - np.float32(mn)
    q = np.rint(d.astype(np.float64) * np.float64(inv))
    q = np.minimum(q, qmax).astype(np.uint8)
    return sh, mn, q


def numpy_dequantize(q, sh, zh):
    # code*scale + zero is exact in float64 (8 + 11 bits against a span of < 53 bits),
    # so one rounding to float32 equals a float32 fma
    exact = q.astype(np.float64) * np.float64(sh) + np.float64(zh)
    return exact.astype(np.float32).astype(np.float16)


def random_group(rng, n, kind):
    if kind == "normal":
        x = rng.standard_normal(n)
    elif kind == "outlier":
        x = rng.standard_normal(n)
        x[rng.integers(0, n)] *= 40
    elif kind == "small":
        x = rng.standard_normal(n) * 1e-4
    elif kind == "subnormal":
        x = rng.standard_normal(n) * 3e-7
    elif kind == "large":
        x = rng.standard_normal(n) * 8000
    elif kind == "offset":
        x = rng.standard_normal(n) * 0.01 + 100
    else:
        raise ValueError(kind)
    return np.clip(x, -65000, 65000).astype(np.float16)


KINDS = ["normal", "outlier", "small", "subnormal", "large", "offset"]


@pytest.mark.parametrize("width", [2, 4, 8])
@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("n", [32, 64, 128])
def test_group_matches_numpy_ieee(width, kind, n):
    rng = np.random.default_rng(width * 1000 + n + 17 * KINDS.index(kind))
    for _ in range(40):
        x = random_group(rng, n, kind)
        sh, zh, q = ref.quantize_group(x, width)
        wsh, wzh, wq = numpy_quantize(x, width)
        assert sh == wsh.view(np.uint16)
        assert zh == wzh.view(np.uint16)
        assert np.array_equal(q, wq)
        got = ref.dequantize_group(q, sh, zh)
        want = numpy_dequantize(q, wsh, wzh).view(np.uint16)
        assert np.array_equal(got, want)


@pytest.mark.parametrize("width", [2, 4, 8])
def test_on_grid_values_round_trip_exactly(width):
    """x_i = z + k_i*s with s a power of two: scale found exactly, codes = k_i, decode = input."""
    qmax = (1 << width) - 1
    rng = np.random.default_rng(11 + width)
    for e in [-10, -6, -3, 0, 2, 4]:
        s = 2.0 ** e
        for m in [-37, -1, 0, 3, 20]:
            k = rng.integers(0, qmax + 1, size=32)
            k[0], k[1] = 0, qmax
            rng.shuffle(k)
            x = ((m + k) * s).astype(np.float16)
            assert np.array_equal(x.astype(np.float64), (m + k) * s)  # fixture itself is exact in fp16
            sh, zh, q = ref.quantize_group(x, width)
            assert f16(sh) == np.float16(s)
            assert f16(zh) == np.float16(m * s)
            assert np.array_equal(q, k.astype(np.uint8))
            assert np.array_equal(ref.dequantize_group(q, sh, zh), x.view(np.uint16))


def ulp16(v):
    v = abs(float(v))
    if v < 2.0 ** -14:
        return 2.0 ** -24
    e = int(np.floor(np.log2(v)))
    return 2.0 ** (e - 10)


@pytest.mark.parametrize("width", [2, 4, 8])
@pytest.mark.parametrize("kind", ["normal", "outlier", "small", "large", "offset"])
def test_error_bound_half_a_step(width, kind):
    """|x - decode| <= scale/2 + half an fp16 ulp of the result + rounding slack (normal scales)."""
    rng = np.random.default_rng(100 + width)
    for _ in range(60):
        x = random_group(rng, 32, kind)
        sh, zh, q = ref.quantize_group(x, width)
        s = float(f16(sh))
        if s < 2.0 ** -14:
            continue
        y = ref.dequantize_group(q, sh, zh).view(np.float16)
        mn = float(f16(zh))
        for xi, yi in zip(x.astype(np.float64), y.astype(np.float64)):
            bound = s / 2 + ulp16(yi) / 2 + 2.0 ** -22 * abs(xi - mn) + 2.0 ** -24 * abs(yi)
            assert abs(xi - yi) <= bound * (1 + 1e-12)


@pytest.mark.parametrize("width", [2, 4, 8])
def test_endpoints(width):
    qmax = (1 << width) - 1
    rng = np.random.default_rng(width)
    for kind in KINDS:
        for _ in range(20):
            x = random_group(rng, 32, kind)
            sh, zh, q = ref.quantize_group(x, width)
            keys = order_key(x.view(np.uint16))
            imin, imax = int(np.argmin(keys)), int(np.argmax(keys))
            assert zh == x.view(np.uint16)[imin]
            assert q[imin] == 0
            assert ref.dequantize_group(q[imin:imin + 1], sh, zh)[0] == zh
            if f16(sh) >= np.float16(2.0 ** -14):
                assert q[imax] == qmax


def test_degenerate_groups():
    # constant group: scale 0, all codes 0, decode returns the constant
    x = np.full(32, 1.25, dtype=np.float16)
    sh, zh, q = ref.quantize_group(x, 4)
    assert sh == 0 and zh == x.view(np.uint16)[0] and not q.any()
    assert np.array_equal(ref.dequantize_group(q, sh, zh), x.view(np.uint16))
    # range so small that the fp16 scale rounds to zero (2^-24 / 255 < 2^-25)
    x = np.zeros(32, dtype=np.uint16)
    x[5] = 1  # smallest subnormal
    sh, zh, q = ref.quantize_group(x, 8)
    assert sh == 0 and not q.any()
    # -0 sorts below +0: zero point must be -0
    x = np.zeros(32, dtype=np.uint16)
    x[7] = 0x8000
    sh, zh, q = ref.quantize_group(x, 2)
    assert zh == 0x8000 and sh == 0 and not q.any()
    x = np.full(32, 0x8000, dtype=np.uint16)
    x[3] = 0
    sh, zh, q = ref.quantize_group(x, 2)
    assert zh == 0x8000


def test_subnormal_scale_needs_the_clamp():
    # range 3 * 2^-24 at 2 bits: exact step 2^-24, fine.  range 4 * 2^-24 at 2 bits: step 4/3 ulp
    # rounds to 1 ulp, the top value would land on code 4 without the clamp.
    x = np.zeros(32, dtype=np.uint16)
    x[1] = 4
    sh, zh, q = ref.quantize_group(x, 2)
    assert sh == 1 and q[1] == 3 and q.max() == 3


@pytest.mark.parametrize("width", [2, 4])
def test_brute_force_nearest_code_in_exact_arithmetic(width):
    """Tiny groups: the chosen code is (one of) the nearest grid points z + q*s in exact rationals."""
    qmax = (1 << width) - 1
    rng = np.random.default_rng(77 + width)
    checked = 0
    for kind in ["normal", "outlier", "offset", "small"]:
        for _ in range(25):
            x = random_group(rng, 8, kind)
            sh, zh, q = ref.quantize_group(x, width)
            s = Fraction(float(f16(sh)))
            z = Fraction(float(f16(zh)))
            if s == 0:
                continue
            for xi, qi in zip(x.tolist(), q.tolist()):
                xi = Fraction(xi)
                errs = [abs(xi - (z + c * s)) for c in range(qmax + 1)]
                best = min(errs)
                # reciprocal and difference roundings move the decision point by at most s * 2^-20
                assert errs[qi] <= best + s / (1 << 20)
                if sum(1 for e in errs if e <= best + s / (1 << 20)) == 1:
                    assert errs[qi] == best
                    checked += 1
    assert checked > 300


def test_exact_ties_round_to_even_code():
    # scale 1, zero 0, values k + 0.5 are exact fp16: ties go to the even code
    x = np.array([0, 15, 0.5, 1.5, 2.5, 3.5, 6.5, 13.5] + [0] * 24, dtype=np.float16)
    sh, zh, q = ref.quantize_group(x, 4)
    assert f16(sh) == np.float16(1.0)
    assert q[:8].tolist() == [0, 15, 0, 2, 2, 4, 6, 14]
