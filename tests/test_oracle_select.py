"""Pins for the oracle's decay + selection + index build (paper Sec. 3.1, 3.3, Algorithm 1):
the paper's worked example, the StreamLLM special case, brute force, a library sort,
invariants and the decay closed form.  CPU only."""
import itertools
import os

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from helpers import read_golden

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def P(ref, n_sink, n_topk, n_recent, decay=1.0):
    return ref.Policy(n_sink, n_topk, n_recent, decay)


# ---------------------------------------------------------------- the paper's own example
def test_worked_example_of_in_cache_positions(ref):
    g = read_golden(os.path.join(GOLDEN, "kept_positions_example.txt"))
    n = g["n_cand"]
    E = np.full((1, n), 1.0, dtype=np.float32)
    E[0, 5], E[0, 7] = 9.0, 8.0                       # the two high-entropy middle slots
    E[0, 0] = 0.0                                     # a sink stays whatever its score
    E[0, 12] = 0.0                                    # and so does a recent slot
    E[0, 11] = 100.0                                  # a recent slot must not use up one of the k
    kept, out = ref.decay_select(E, n_held=n - 3, n_new=3, policy=P(ref, g["n_sink"], g["n_topk"], g["n_recent"]))
    assert kept[0].tolist() == g["kept"]
    # slot j of the compacted cache is in-cache position j
    assert list(range(len(g["kept"]))) == g["in_cache_positions"]
    np.testing.assert_array_equal(out[0], E[0, g["kept"]])


def test_budget_identities_of_the_experiments(ref):
    with open(os.path.join(GOLDEN, "budgets.txt")) as f:
        rows = [[int(x) for x in l.split()] for l in f if l.strip() and not l.startswith("#")]
    rng = np.random.default_rng(0)
    for cache, n_sink, n_ent, n_rec in rows:
        assert n_sink + n_ent + n_rec == cache
        n_cand = cache + 57
        E = rng.gamma(2.0, 2.0, (1, n_cand)).astype(np.float32)
        kept, _ = ref.decay_select(E, n_cand - 57, 57, P(ref, n_sink, n_ent, n_rec, 0.7))
        assert kept.shape == (1, cache)
        assert kept[0, :n_sink].tolist() == list(range(n_sink))


# ---------------------------------------------------------------- special cases
def test_k_zero_is_streamllm(ref):
    # sink + recent only, irrespective of scores (Sec. 3.1)
    rng = np.random.default_rng(3)
    E = rng.standard_normal((2, 50)).astype(np.float32)
    kept, _ = ref.decay_select(E, 40, 10, P(ref, 4, 0, 6))
    want = list(range(4)) + list(range(44, 50))
    assert kept[0].tolist() == want and kept[1].tolist() == want


def test_no_recent_no_sink(ref):
    E = np.array([[1, 5, 2, 4, 3, 0]], dtype=np.float32)
    kept, out = ref.decay_select(E, 6, 0, P(ref, 0, 3, 0))
    assert kept[0].tolist() == [1, 3, 4]
    assert out[0].tolist() == [5, 4, 3]
    kept, _ = ref.decay_select(E, 3, 3, P(ref, 0, 0, 2))     # sliding window
    assert kept[0].tolist() == [4, 5]


def test_at_or_under_budget_keeps_everything_but_still_decays(ref):
    E = np.array([[4, 3, 2, 1, 7, 7]], dtype=np.float32)
    for budget_k in (2, 3):                                    # n_cand == budget and n_cand < budget
        kept, out = ref.decay_select(E, 4, 2, P(ref, 2, budget_k, 2, 0.5))
        assert kept[0].tolist() == [0, 1, 2, 3, 4, 5]
        assert out[0].tolist() == [2, 1.5, 1, 0.5, 7, 7]       # held halved, new untouched


def test_all_ties_take_the_lowest_middle_slots(ref):
    E = np.full((1, 40), 2.5, dtype=np.float32)
    kept, _ = ref.decay_select(E, 30, 10, P(ref, 3, 5, 4))
    assert kept[0].tolist() == [0, 1, 2] + [3, 4, 5, 6, 7] + [36, 37, 38, 39]


def test_ties_straddling_the_kth_boundary(ref):
    #            0  1  2  3  4  5  6  7  8  9
    E = np.array([[0, 5, 3, 9, 3, 3, 1, 3, 0, 0]], dtype=np.float32)
    kept, _ = ref.decay_select(E, 10, 0, P(ref, 1, 4, 2))     # middle = 1..7, top-4: 9,5 and two of the 3s
    assert kept[0].tolist() == [0, 1, 2, 3, 4, 8, 9]


def test_signed_zero_and_negative_scores(ref):
    E = np.array([[-0.0, 0.0, -1.0, -0.0, 0.0, -2.0]], dtype=np.float32)
    kept, _ = ref.decay_select(E, 6, 0, P(ref, 0, 3, 0))
    assert kept[0].tolist() == [0, 1, 3]                      # the zeros tie (+0 == -0): lowest slots first
    kept, _ = ref.decay_select(E, 6, 0, P(ref, 0, 5, 0))
    assert kept[0].tolist() == [0, 1, 2, 3, 4]                # -1 beats -2


def test_nan_and_inf_order(ref):
    pos_nan = np.array([0x7FC00000], dtype=np.uint32).view(np.float32)[0]
    neg_nan = np.array([0xFFC00000], dtype=np.uint32).view(np.float32)[0]
    E = np.array([[1.0, np.inf, pos_nan, -np.inf, neg_nan, 2.0]], dtype=np.float32)
    order = []
    for k in range(1, 7):
        kept, _ = ref.decay_select(E, 0, 6, P(ref, 0, k, 0))
        if k < 6:
            new = set(kept[0].tolist()) - set(order)
            order.append(new.pop())
    assert order == [2, 1, 5, 0, 3]                            # +NaN > +inf > 2 > 1 > -inf (> -NaN)


# ---------------------------------------------------------------- decay
def test_decay_is_one_binary32_multiply_on_held_only(ref):
    rng = np.random.default_rng(5)
    E = rng.gamma(2.0, 2.0, (3, 64)).astype(np.float32)
    E[0, 0] = np.float32(1e-41)                               # a denormal stays a denormal
    eta = np.float32(0.9)
    kept, out = ref.decay_select(E, 48, 16, P(ref, 4, 100, 8, float(eta)))
    want = E.copy()
    want[:, :48] = E[:, :48] * eta                             # numpy float32 multiply: one rounding
    np.testing.assert_array_equal(out.view(np.uint32), want.view(np.uint32))
    assert out[0, 0] != 0.0


def test_decay_applied_once_per_turn_sentinel(ref):
    # a sentinel of exactly 1.0 kept for T turns holds the T-fold binary32 product of eta
    eta = np.float32(0.85)
    pol = P(ref, 1, 2, 1, float(eta))
    E = np.array([[1.0, 0.5, 0.25, 0.125]], dtype=np.float32)   # slot 0 is a sink: never evicted
    want = np.float32(1.0)
    for turn in range(12):
        cand = np.concatenate([E, np.full((1, 3), 0.01, dtype=np.float32)], axis=1)
        kept, E = ref.decay_select(cand, E.shape[1], 3, pol)
        want = np.float32(want * eta)
        assert E[0, 0] == want
        assert E.shape[1] == 4


@pytest.mark.parametrize("eta,e0,c", [(0.9, 6.0, 2.0), (0.7, 5.0, 1.0), (0.5, 9.0, 0.3)])
def test_forgetting_horizon(ref, eta, e0, c):
    # One early token with score e0; every later turn brings more than k + n_recent tokens that
    # all score c < e0.  With eta < 1 the early token leaves the cache at the first turn T* at
    # which its T*-fold decayed score drops below c (Sec. 3.3: older key information is
    # forgotten); with eta = 1 it never leaves (Sec. 5, decay-ratio study: only eta = 1 keeps
    # the early item).
    pol = P(ref, 2, 4, 3, eta)
    n_new = 10
    def run(decay, turns=40):
        p = ref.Policy(pol.n_sink, pol.n_topk, pol.n_recent, decay)
        E = np.array([[0.1, 0.1, e0]], dtype=np.float32)
        tag = np.array([[-1, -1, 7]])                          # 7 marks the early token
        for t in range(1, turns + 1):
            cand = np.concatenate([E, np.full((1, n_new), c, dtype=np.float32)], axis=1)
            ctag = np.concatenate([tag, np.zeros((1, n_new), dtype=int)], axis=1)
            kept, E = ref.decay_select(cand, E.shape[1], n_new, p)
            tag = ctag[:, kept[0]]
            if 7 not in tag:
                return t
        return None
    v, T_star = np.float32(e0), None
    for t in range(1, 41):
        v = np.float32(v * np.float32(eta))
        if v < np.float32(c):
            T_star = t
            break
    assert run(eta) == T_star
    assert run(1.0) is None


# ---------------------------------------------------------------- brute force
def best_subsets(E, mid, k):
    """Every k-subset S of the middle slots such that no excluded slot beats an included one
    under (score descending, slot ascending)."""
    def beats(a, b):
        return E[a] > E[b] or (E[a] == E[b] and a < b)
    good = []
    for S in itertools.combinations(mid, k):
        Sset = set(S)
        if not any(beats(o, i) for o in mid if o not in Sset for i in S):
            good.append(S)
    return good


@pytest.mark.parametrize("seed", range(6))
def test_against_subset_enumeration(ref, seed):
    rng = np.random.default_rng(seed)
    n_cand, n_sink, k, n_recent = 12, 2, 4, 2
    E = rng.integers(0, 4, (1, n_cand)).astype(np.float32)     # few distinct values: many ties
    kept, _ = ref.decay_select(E, n_cand, 0, P(ref, n_sink, k, n_recent))
    mid = list(range(n_sink, n_cand - n_recent))
    subsets = best_subsets(E[0], mid, k)
    assert len(subsets) == 1                                   # the order is total, so the answer is unique
    want = list(range(n_sink)) + list(subsets[0]) + list(range(n_cand - n_recent, n_cand))
    assert kept[0].tolist() == sorted(want)


@settings(max_examples=120, deadline=None)
@given(st.data())
def test_invariants_and_library_sort(ref, data):
    n_streams = data.draw(st.integers(1, 3))
    n_held = data.draw(st.integers(0, 120))
    n_new = data.draw(st.integers(0, 60))
    n_sink = data.draw(st.integers(0, 6))
    k = data.draw(st.integers(0, 40))
    n_recent = data.draw(st.integers(0, 30))
    levels = data.draw(st.sampled_from([3, 17, 100000]))
    eta = data.draw(st.sampled_from([1.0, 0.9, 0.5]))
    seed = data.draw(st.integers(0, 2**31))
    n_cand = n_held + n_new
    if n_cand == 0:
        return
    rng = np.random.default_rng(seed)
    E = (rng.integers(0, levels, (n_streams, n_cand)) / 7.0).astype(np.float32)
    pol = P(ref, n_sink, k, n_recent, eta)
    kept, out = ref.decay_select(E, n_held, n_new, pol)
    budget = n_sink + k + n_recent
    D = E.copy()
    D[:, :n_held] = E[:, :n_held] * np.float32(eta)
    assert kept.shape == (n_streams, min(n_cand, budget))
    for s in range(n_streams):
        ks = kept[s]
        assert (np.diff(ks) > 0).all()                         # strictly ascending
        np.testing.assert_array_equal(out[s], D[s, ks])        # E <- E[Id] on the decayed values
        if n_cand <= budget:
            assert ks.tolist() == list(range(n_cand))
            continue
        kset = set(ks.tolist())
        assert set(range(n_sink)) <= kset
        assert set(range(n_cand - n_recent, n_cand)) <= kset
        mid = np.arange(n_sink, n_cand - n_recent)
        order = np.lexsort((mid, -D[s, mid].astype(np.float64)))   # library sort: score desc, slot asc
        want_mid = set(mid[order[:k]].tolist())
        assert kset - set(range(n_sink)) - set(range(n_cand - n_recent, n_cand)) == want_mid
