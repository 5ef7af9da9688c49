"""Pins for the oracle's baseline policies (paper Sec. 4.1: StreamLLM, IntervalLLM, RandomLLM):
published known-answer vectors for the generator, hand-worked interval combs, and the properties
a uniformly random subset must have.  CPU only."""
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_philox_known_answers(ref):
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as f:
        rows = [[int(x, 16) for x in l.split()] for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        assert ref.philox4x32_10(r[0:4], r[4:6]) == r[6:10]


def test_stream_policy_is_sink_plus_recent(ref):
    kept = ref.baseline_select(ref.STREAM, 2, 50, ref.Policy(4, 999, 6, 0.0))
    want = list(range(4)) + list(range(44, 50))
    assert kept.shape == (2, 10) and kept[0].tolist() == want and kept[1].tolist() == want
    # identical to the entropy policy with k = 0 (Sec. 3.1)
    E = np.random.default_rng(0).standard_normal((2, 50)).astype(np.float32)
    ki, _ = ref.decay_select(E, 50, 0, ref.Policy(4, 0, 6, 1.0))
    np.testing.assert_array_equal(kept, ki)


def test_interval_comb_by_hand(ref):
    # 4 sinks, middle = slots 4..23 (M = 20), k = 5 -> interval 4, anchored at the newest middle slot 23
    kept = ref.baseline_select(ref.INTERVAL, 1, 26, ref.Policy(4, 5, 2, 0.0))
    assert kept[0].tolist() == [0, 1, 2, 3, 7, 11, 15, 19, 23, 24, 25]
    # M = 23, k = 5 -> interval floor(23/5) = 4: 26, 22, 18, 14, 10
    kept = ref.baseline_select(ref.INTERVAL, 1, 29, ref.Policy(4, 5, 2, 0.0))
    assert kept[0].tolist() == [0, 1, 2, 3, 10, 14, 18, 22, 26, 27, 28]
    # M < 2k -> interval 1: the k newest middle slots
    kept = ref.baseline_select(ref.INTERVAL, 1, 20, ref.Policy(2, 8, 3, 0.0))
    assert kept[0].tolist() == [0, 1] + list(range(9, 17)) + [17, 18, 19]
    # the paper's setting, cache 1024 = 4 + 1020 + 0 with 54 new tokens: interval floor(1074/1020) = 1
    kept = ref.baseline_select(ref.INTERVAL, 1, 1078, ref.Policy(4, 1020, 0, 0.0))
    assert kept[0].tolist() == [0, 1, 2, 3] + list(range(58, 1078))


def test_under_budget_keeps_everything(ref):
    for kind in (ref.STREAM, ref.INTERVAL, ref.RANDOM):
        pol = ref.Policy(4, 20, 8, 0.0)
        n_cand = 12 if kind == ref.STREAM else 30
        kept = ref.baseline_select(kind, 2, n_cand, pol, seed=3, turn=1)
        assert kept[0].tolist() == list(range(n_cand))


def test_random_subset_properties(ref):
    pol = ref.Policy(4, 100, 16, 0.0)
    n_cand = 600
    a = ref.baseline_select(ref.RANDOM, 3, n_cand, pol, seed=11, turn=5)
    assert a.shape == (3, 120)
    for s in range(3):
        assert (np.diff(a[s]) > 0).all()
        assert a[s, :4].tolist() == [0, 1, 2, 3] and a[s, -16:].tolist() == list(range(584, 600))
        assert ((a[s, 4:104] >= 4) & (a[s, 4:104] < 584)).all()
    assert not np.array_equal(a[0], a[1])                      # streams draw independently
    np.testing.assert_array_equal(a, ref.baseline_select(ref.RANDOM, 3, n_cand, pol, seed=11, turn=5))
    assert not np.array_equal(a, ref.baseline_select(ref.RANDOM, 3, n_cand, pol, seed=12, turn=5))
    assert not np.array_equal(a, ref.baseline_select(ref.RANDOM, 3, n_cand, pol, seed=11, turn=6))
    assert not np.array_equal(a, ref.baseline_select(ref.RANDOM, 3, n_cand, pol, seed=11 + (1 << 32), turn=5))
    assert not np.array_equal(a, ref.baseline_select(ref.RANDOM, 3, n_cand, pol, seed=11, turn=5 + (1 << 32)))


def test_random_subset_follows_the_published_generator(ref):
    # rebuild the subset from the generator's outputs alone: slot i of stream s draws word 0 of
    # philox(ctr = {i, s, turn_lo, turn_hi}, key = {seed_lo, seed_hi}); the k largest draws stay
    pol = ref.Policy(2, 7, 3, 0.0)
    n_cand, seed, turn = 40, (5 << 32) | 9, (1 << 32) | 77
    kept = ref.baseline_select(ref.RANDOM, 2, n_cand, pol, seed=seed, turn=turn)
    for s in range(2):
        draws = {i: ref.philox4x32_10([i, s, turn & 0xffffffff, turn >> 32], [seed & 0xffffffff, seed >> 32])[0]
                 for i in range(2, 37)}
        top = sorted(draws, key=lambda i: (-draws[i], i))[:7]
        assert kept[s].tolist() == [0, 1] + sorted(top) + [37, 38, 39]


def test_random_subset_is_uniform(ref):
    # every middle slot is kept with probability k / M: 400 draws of 10 out of 40
    pol = ref.Policy(0, 10, 0, 0.0)
    counts = np.zeros(40)
    for turn in range(400):
        counts[ref.baseline_select(ref.RANDOM, 1, 40, pol, seed=1, turn=turn)[0]] += 1
    # binomial(400, 1/4): mean 100, sd 8.7; all 40 slots within 4.5 sd
    assert (np.abs(counts - 100) < 39).all(), counts
