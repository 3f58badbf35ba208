"""Pins of the controller oracle (network scores and objective-greedy allocator) against values fixed
by arithmetic, closed forms, brute force and a float64 library matmul; no GPU."""
import itertools
from fractions import Fraction

import numpy as np
import pytest

import qkv_synth
from oracle import ref

F32 = np.float32


def zero_net():
    return np.zeros((64, 6), F32), np.zeros(64, F32), np.zeros(64, F32)


# ---------------------------------------------------------------- network (paper Sec. 4.1.2)

def test_parameter_count_is_512():
    w1, b1, w2 = zero_net()
    assert w1.size + b1.size + w2.size == 512


def test_hand_computed_small_integers():
    # all products and sums are small integers, exact in fp32, worked out by hand:
    # unit 0: 1 + 1*2 + 2*3 = 9 -> relu 9, times 2 -> 18;  unit 1: -20 + 1*1 + 2*1 = -17 -> relu 0;
    # unit 5: 0.5 + 3*(-1)*(-1) = 3.5 -> times 4 -> 14.  Sum 32.
    w1, b1, w2 = zero_net()
    w1[0, 0], w1[0, 1], b1[0], w2[0] = 2, 3, 1, 2
    w1[1, 0], w1[1, 1], b1[1], w2[1] = 1, 1, -20, 1000
    w1[5, 5], b1[5], w2[5] = -3, 0.5, 4
    x = np.array([[1, 2, 0, 0, 0, -1]], F32)
    assert ref.controller_scores(x, w1, b1, w2)[0] == F32(32.0)


def test_hidden_unit_is_one_fused_chain_from_the_bias():
    # x0*w = (1+2^-12)^2 = 1 + 2^-11 + 2^-24; fused with the bias -1 the exact 2^-11 + 2^-24 survives,
    # a separately rounded product (tie to even -> 1 + 2^-11) would leave 2^-11 only
    w1, b1, w2 = zero_net()
    a = F32(1 + 2.0 ** -12)
    w1[0, 0], b1[0], w2[0] = a, -1, 1
    x = np.zeros((1, 6), F32)
    x[0, 0] = a
    assert ref.controller_scores(x, w1, b1, w2)[0] == F32(2.0 ** -11 + 2.0 ** -24)


def test_output_accumulates_units_in_order_from_zero():
    # hidden values 2^24, 1, 2^24 with output weights 1, 1, -1: in order, 2^24 + 1 rounds back to 2^24
    # (tie to even) and the sum ends at 0; any other order or a wider accumulator gives 1
    w1, b1, w2 = zero_net()
    b1[0], b1[1], b1[2] = 2.0 ** 24, 1, 2.0 ** 24
    w2[0], w2[1], w2[2] = 1, 1, -1
    assert ref.controller_scores(np.zeros((1, 6), F32), w1, b1, w2)[0] == F32(0.0)
    b1[0], b1[1], b1[2] = 1, 2.0 ** 24, 2.0 ** 24       # the same terms, 1 first: now it survives... as 2^24+1 ties to 2^24
    w2[0], w2[1], w2[2] = 1, 1, -1
    assert ref.controller_scores(np.zeros((1, 6), F32), w1, b1, w2)[0] == F32(0.0)
    b1[0], b1[1], b1[2] = 2.0 ** 24, 2.0 ** 24, 1        # cancel first, then add 1
    w2[0], w2[1], w2[2] = 1, -1, 1
    assert ref.controller_scores(np.zeros((1, 6), F32), w1, b1, w2)[0] == F32(1.0)


def test_relu_blocks_negative_units_and_nan():
    w1, b1, w2 = zero_net()
    b1[:] = -1.0
    w2[:] = 1e30
    assert ref.controller_scores(np.ones((3, 6), F32) * 0.1, w1, b1, w2).tolist() == [0.0, 0.0, 0.0]
    b1[:] = 0
    b1[7] = np.nan
    b1[8] = 2
    w2[:] = 1
    assert ref.controller_scores(np.zeros((1, 6), F32), w1, b1, w2)[0] == F32(2.0)


def test_matches_float64_matmul():
    T = 500
    x = qkv_synth.make_features(T, 11).numpy()
    w1, b1, w2 = [a.numpy() for a in qkv_synth.make_controller(12)]
    got = ref.controller_scores(x, w1, b1, w2).astype(np.float64)
    h = np.maximum(x.astype(np.float64) @ w1.astype(np.float64).T + b1.astype(np.float64), 0.0)
    want = h @ w2.astype(np.float64)
    assert np.max(np.abs(got - want)) <= 64 * 2.0 ** -23 * np.max(np.abs(h) @ np.abs(w2.astype(np.float64)))
    assert np.max(np.abs(got - want)) > 0          # it is fp32, not a float64 copy


def test_power_of_two_scaling_of_output_weights_is_exact():
    x = qkv_synth.make_features(64, 13).numpy()
    w1, b1, w2 = [a.numpy() for a in qkv_synth.make_controller(14)]
    s = ref.controller_scores(x, w1, b1, w2)
    assert np.array_equal(ref.controller_scores(x, w1, b1, w2 * F32(8)), s * F32(8))


def test_each_token_stands_alone():
    x = qkv_synth.make_features(40, 15).numpy()
    w1, b1, w2 = [a.numpy() for a in qkv_synth.make_controller(16)]
    s = ref.controller_scores(x, w1, b1, w2)
    for t in (0, 17, 39):
        assert ref.controller_scores(x[t:t + 1], w1, b1, w2)[0] == s[t]


def test_features_recipe():
    f = qkv_synth.make_features(1000, 3).numpy()
    assert f.shape == (1000, 6) and f.dtype == np.float32
    assert set(np.unique(f[:, 5]).tolist()) <= {0.0, 0.5, 1.0}
    assert np.all(f[:, :4] > 0) and np.all(f[:, :4] < 1)
    assert np.all(f[f[:, 5] > 0, 4] >= 0.5)
    for s in range(0, 1000, 64):
        assert len(np.unique(f[s:s + 64, 5])) == 1


# ---------------------------------------------------------------- objective-greedy allocator (paper Sec. 3.3)

EPS = {2: Fraction(1, 3), 4: Fraction(1, 15), 8: Fraction(1, 255), 16: Fraction(1, 65535)}


def objective(bits, scores):
    return sum(EPS[int(b)] * Fraction(float(s)) for b, s in zip(bits, scores))


def incremental_greedy(scores, budget_bits):
    """The greedy rule taken one step at a time in exact rationals: always the upgrade with the largest
    gain per bit (ties: lower level, then lower index); stop when it does not fit."""
    T = len(scores)
    bits = [2] * T
    spare = budget_bits - 2 * T
    while True:
        best = None
        for t in range(T):
            b = bits[t]
            if b == 16:
                continue
            gain = Fraction(max(float(scores[t]), 0.0)) * (EPS[b] - EPS[2 * b]) / b      # the upgrade costs b bits
            key = (-gain, b, t)
            if best is None or key < best[0]:
                best = (key, t, b)
        if best is None or best[2] > spare:
            return bits
        spare -= best[2]
        bits[best[1]] *= 2


@pytest.mark.parametrize("budget", [2.0, 2.5, 3.0, 4.0, 5.5, 8.0, 12.0, 16.0])
def test_equals_step_by_step_greedy(budget):
    # scores on a coarse grid far from fp32 near-ties between different tokens' products
    rng = np.random.default_rng(5)
    scores = rng.permutation(np.arange(1, 41)).astype(F32) * F32(0.37)
    bits, counts = ref.assign_bits_greedy(scores, budget)
    want = incremental_greedy(scores, int(round(budget * 1000)) * 40 // 1000)
    assert bits.tolist() == want
    assert counts.tolist() == [want.count(w) for w in (2, 4, 8, 16)]


def test_optimal_for_the_bits_it_spends():
    # brute force over all 4^6 assignments: nothing that costs at most what the greedy prefix spent
    # has a smaller objective
    scores = np.array([5, 1, 9, 3, 7, 2], F32)
    for budget in (2.4, 3.0, 3.7, 4.4, 6.0, 9.0):
        bits, _ = ref.assign_bits_greedy(scores, budget)
        spent = int(bits.sum())
        assert spent <= int(budget * 6 + 1e-9)
        mine = objective(bits, scores)
        for other in itertools.product((2, 4, 8, 16), repeat=6):
            if sum(other) <= spent:
                assert objective(other, scores) >= mine


def test_closed_form_on_uniform_scores():
    # scores i/T: a threshold lam on the gain per bit gives fractions 1 - 7.5 lam with >= 4 bits and
    # 1 - 63.75 lam with >= 8; at budget 4 the spend 2 + 2 f4 + 4 f8 = 4 gives lam = 4/270:
    # 1/9 of the tokens at 2 bits, 5/6 at 4, 1/18 at 8, none at 16
    T = 18000
    scores = (np.arange(T, dtype=np.float64) + 0.5) / T
    bits, counts = ref.assign_bits_greedy(scores.astype(F32), 4.0)
    assert abs(counts[0] - T / 9) <= 3 and abs(counts[1] - T * 5 / 6) <= 3 and abs(counts[2] - T / 18) <= 3 and counts[3] == 0
    assert np.all(np.diff(bits.astype(int)) >= 0)                  # monotone in the score
    assert 4 * T - 8 < int(bits.astype(np.int64).sum()) <= 4 * T


def test_budget_ends_and_errors():
    s = qkv_synth.make_scores(300, 21).numpy()
    assert ref.assign_bits_greedy(s, 2.0)[1].tolist() == [300, 0, 0, 0]
    assert ref.assign_bits_greedy(s, 16.0)[1].tolist() == [0, 0, 0, 300]
    assert ref.assign_bits_greedy(s, 2.0 + 2.0 / 300)[1].tolist() == [299, 1, 0, 0]
    assert ref.assign_bits_greedy(s, 2.0 + 2.0 / 300)[0][int(np.argmax(s))] == 4
    for bad in (1.9, 16.5, float("nan")):
        with pytest.raises(ref.OracleError):
            ref.assign_bits_greedy(s, bad)


def test_ties_zero_and_negative_scores():
    # equal scores: level first, then index.  10 tokens, budget 3.0 -> 10 spare bits -> the first five
    # tokens go to 4 bits (a 4->8 upgrade of token 0 ranks after every 2->4 upgrade)
    bits, _ = ref.assign_bits_greedy(np.ones(10, F32), 3.0)
    assert bits.tolist() == [4] * 5 + [2] * 5
    # all 2->4 taken (20 bits), then 4->8 by index with the remaining 12
    bits, _ = ref.assign_bits_greedy(np.ones(10, F32), 5.2)
    assert bits.tolist() == [8] * 3 + [4] * 7
    # negative and NaN scores count as zero: they rank behind every upgrade of a positive score, level
    # first, then index.  21 bits -> 9 spare: t2 2->4, t5 2->4, t2 4->8, then t5 4->8 does not fit
    s = np.array([-5, 0, 3, np.nan, -0.0, 2], F32)
    bits, _ = ref.assign_bits_greedy(s, 3.5)
    assert bits.tolist() == [2, 2, 8, 2, 2, 4]
    # 46 bits -> 34 spare: 28 take tokens 2 and 5 to 16 bits, the other 6 the first three zero-score tokens to 4
    bits, _ = ref.assign_bits_greedy(s, 7.667)
    assert bits.tolist() == [4, 4, 16, 4, 2, 16]


def test_prefix_stops_at_the_first_upgrade_that_does_not_fit():
    # scores 100, 1, 1: order is t0 2->4 (gain 13.3/bit), t0 4->8 (1.57/bit), then t1 2->4 (0.133/bit) ...
    # with 4 spare bits t0 goes to 4 bits, its 4->8 upgrade (4 bits) does not fit in the 2 left, and the
    # cheaper upgrades behind it are not taken either
    bits, _ = ref.assign_bits_greedy(np.array([100, 1, 1], F32), 2.0 + 4.0 / 3)
    assert bits.tolist() == [4, 2, 2]


def test_sum_of_bits_within_budget_and_monotone():
    for seed, budget in ((31, 2.7), (32, 3.3), (33, 6.1), (34, 10.0)):
        s = qkv_synth.make_scores(777, seed).numpy()
        bits, counts = ref.assign_bits_greedy(s, budget)
        assert int(bits.astype(np.int64).sum()) <= int(round(budget * 1000)) * 777 // 1000
        assert counts.sum() == 777
        order = np.argsort(-s, kind="stable")
        assert np.all(np.diff(bits[order].astype(int)) <= 0)
