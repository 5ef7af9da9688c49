"""Pins for the oracle's token entropy taken straight from the language-model head
(paper Sec. 3.2: the probabilities are the model's own softmax output, so the logits are
hidden @ weight.T): float64 library matmul + logsumexp, closed forms, reduction to the
pinned logits-based score, layout cases.  CPU only."""
import math

import numpy as np
import pytest
import torch
from scipy.special import logsumexp

from helpers import logits_f64, to_np


def bf16_bits(x: np.ndarray) -> np.ndarray:
    return to_np(torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16))


def as_dtype(x, dtype):
    return x.astype(np.float32) if dtype == "f32" else (bf16_bits(x) if dtype == "bf16" else x.astype(np.float16))


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_matches_float64_library_matmul_and_logsumexp(ref, dtype):
    rng = np.random.default_rng(11)
    n, d, V = 13, 96, 517                                   # all different: a transposed operand cannot pass
    h = as_dtype(rng.standard_normal((n, d)), dtype)
    w = as_dtype(rng.standard_normal((V, d)) * 0.4, dtype)
    tok = rng.integers(0, V, n).astype(np.int32)
    e = ref.lmhead_score(h, w, tok)
    z = logits_f64(h) @ logits_f64(w).T                      # numpy's float64 matmul
    want = logsumexp(z, axis=1) - z[np.arange(n), tok]
    np.testing.assert_allclose(e, want.astype(np.float32), rtol=3e-7, atol=0)
    ce = torch.nn.functional.cross_entropy(torch.from_numpy(z), torch.from_numpy(tok).long(), reduction="none")
    np.testing.assert_allclose(e, ce.numpy().astype(np.float32), rtol=3e-7, atol=0)


def test_one_hot_hidden_reduces_to_the_logits_score(ref):
    # hidden = unit vector j -> the logits are column j of the weight, exactly: the result must equal the
    # (separately pinned) score of those logits given as a stored row
    rng = np.random.default_rng(12)
    d, V = 24, 300
    w = bf16_bits(rng.standard_normal((V, d)) * 3)
    for j in (0, 7, d - 1):
        h = np.zeros((2, d), dtype=np.float32)
        h[:, j] = 1.0
        hb = bf16_bits(h)
        tok = np.array([5, V - 1], dtype=np.int32)
        e = ref.lmhead_score(hb, w, tok)
        row = np.ascontiguousarray(w[:, j])[None, :].repeat(2, 0)
        np.testing.assert_array_equal(e, ref.score(np.ascontiguousarray(row), tok))


@pytest.mark.parametrize("V,d", [(1000, 16), (4099, 8)])
def test_equal_output_embeddings_give_log_V(ref, V, d):
    rng = np.random.default_rng(13)
    h = rng.standard_normal((3, d)).astype(np.float32)
    w = np.tile(rng.standard_normal((1, d)).astype(np.float32), (V, 1))
    e = ref.lmhead_score(h, w, np.array([0, V // 2, V - 1], dtype=np.int32))
    np.testing.assert_allclose(e, np.float32(math.log(V)), rtol=0, atol=1e-6)
    e0 = ref.lmhead_score(np.zeros((1, d), np.float32), rng.standard_normal((V, d)).astype(np.float32),
                          np.array([3], dtype=np.int32))
    np.testing.assert_allclose(e0, np.float32(math.log(V)), rtol=0, atol=1e-6)   # zero hidden state: uniform


@pytest.mark.parametrize("a", [8.0, -2.0, 0.5])
def test_two_valued_closed_form(ref, a):
    # weight row `hot` = a * u, every other row 0, hidden . u = 1  ->  z = a at hot, 0 elsewhere:
    # e(hot) = log(e^a + V - 1) - a, e(other) = log(e^a + V - 1).  u has power-of-two entries so the
    # products are exact.
    V, d = 777, 8
    u = np.array([1, 0.5, 2, 0.25, 1, 4, 0.5, 1], dtype=np.float64)
    hid = np.zeros(d)
    hid[5] = 0.25                                           # u . hid = u[5] * 0.25 = 1 exactly
    w = np.zeros((V, d), dtype=np.float32)
    hot = 123
    w[hot] = (a * u).astype(np.float32)
    h = np.tile(hid.astype(np.float32), (2, 1))
    e = ref.lmhead_score(h, w, np.array([hot, hot + 1], dtype=np.int32))
    logZ = math.log(math.exp(a) + V - 1)
    np.testing.assert_allclose(e, np.array([logZ - a, logZ], dtype=np.float32), rtol=2e-7, atol=0)


def test_brute_force_loops_on_a_tiny_case(ref):
    # every index written out: rows, vocabulary and model dimension carry different values
    n, d, V = 3, 4, 5
    h = (np.arange(n)[:, None] * 0.5 - np.arange(d)[None, :] * 0.25 + 0.125).astype(np.float32)
    w = (np.arange(V)[:, None] * 0.375 + np.arange(d)[None, :] * np.arange(V)[:, None] * 0.0625 - 0.5).astype(np.float32)
    tok = np.array([4, 0, 2], dtype=np.int32)
    e = ref.lmhead_score(h, w, tok)
    for r in range(n):
        z = [sum(float(h[r, k]) * float(w[v, k]) for k in range(d)) for v in range(V)]
        want = math.log(sum(math.exp(x) for x in z)) - z[tok[r]]
        assert abs(e[r] - want) <= 2e-7 * abs(want)


def test_leading_dimensions_skip_the_padding(ref):
    rng = np.random.default_rng(14)
    n, d, V = 5, 20, 64
    h = np.full((n, 32), 1.0e3, dtype=np.float32)
    w = np.full((V + 3, 48), -1.0e3, dtype=np.float32)
    h[:, :d] = rng.standard_normal((n, d))
    w[:V, :d] = rng.standard_normal((V, d))
    tok = rng.integers(0, V, n).astype(np.int32)
    e = ref.lmhead_score(h, w, tok, d_model=d, vocab=V)
    e_tight = ref.lmhead_score(np.ascontiguousarray(h[:, :d]), np.ascontiguousarray(w[:V, :d]), tok)
    np.testing.assert_array_equal(e, e_tight)


def test_out_of_range_token_and_empty(ref):
    h = np.ones((3, 4), dtype=np.float32)
    w = np.ones((10, 4), dtype=np.float32)
    e = ref.lmhead_score(h, w, np.array([-1, 10, 9], dtype=np.int32))
    assert np.isnan(e[0]) and np.isnan(e[1]) and e[2] == np.float32(math.log(10))
    assert ref.lmhead_score(np.zeros((0, 4), np.float32), w, np.zeros(0, dtype=np.int32)).shape == (0,)
    with pytest.raises(ValueError):
        ref.lmhead_score(h, w, np.zeros(3, dtype=np.int32), d_model=5)
