"""Pins for the oracle's token-entropy score (paper Sec. 3.2): closed forms, a library
routine in float64, invariances and the non-finite cases.  CPU only."""
import math

import numpy as np
import pytest
import torch
from scipy.special import logsumexp

from helpers import logits_f64, to_np
from paper_2405_12528_amd import synth


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    return to_np(torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16))


@pytest.mark.parametrize("V", [1000, 32000, 128256])
@pytest.mark.parametrize("c", [0.0, -3.25, 17.5])
def test_uniform_row_gives_log_V(ref, V, c):
    # all logits equal -> P = 1/V for every token -> e = log V, whatever the constant and the token
    z = np.full((3, V), c, dtype=np.float32)
    tok = np.array([0, V // 2, V - 1], dtype=np.int32)
    e = ref.score(z, tok)
    np.testing.assert_allclose(e, np.float32(math.log(V)), rtol=0, atol=1e-6)
    eb = ref.score(f32_to_bf16_bits(z), tok)
    np.testing.assert_allclose(eb, np.float32(math.log(V)), rtol=0, atol=1e-6)


def test_one_hot_row_gives_zero(ref):
    V = 1000
    z = np.zeros((2, V), dtype=np.float32)
    z[0, 123] = 60.0
    z[1, 999] = 200.0
    e = ref.score(z, np.array([123, 999], dtype=np.int32))
    assert e[0] == 0.0 and e[1] == 0.0          # log(1 + 999 e^-60) rounds to 0 in binary32


@pytest.mark.parametrize("V,a", [(1000, 8.0), (32000, 8.0), (1000, -2.0), (50, 0.5)])
def test_two_valued_row_closed_form(ref, V, a):
    # one logit a, V-1 logits 0:  Z = e^a + V - 1;  e(hot) = log Z - a,  e(other) = log Z.
    # (The Shannon entropy of that row is a different number, so this also fixes the reading
    # "surprisal of the observed token".)
    z = np.zeros((2, V), dtype=np.float32)
    hot = V // 3
    z[:, hot] = a
    tok = np.array([hot, hot + 1], dtype=np.int32)
    e = ref.score(z, tok)
    logZ = math.log(math.exp(a) + V - 1)
    np.testing.assert_allclose(e, np.array([logZ - a, logZ], dtype=np.float32), rtol=1e-7, atol=0)
    p = np.array([math.exp(a)] + [1.0] * (V - 1)) / (math.exp(a) + V - 1)
    shannon = -(p * np.log(p)).sum()
    assert abs(e[0] - shannon) > 1e-3


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_matches_float64_library_log_softmax(ref, dtype):
    rng = np.random.default_rng(1)
    n, V = 37, 2311
    z = (rng.standard_normal((n, V)) * 3.0).astype(np.float32)
    z[::3, rng.integers(0, V)] += 8.0
    zin = z if dtype == "f32" else (f32_to_bf16_bits(z) if dtype == "bf16" else z.astype(np.float16))
    tok = rng.integers(0, V, n).astype(np.int32)
    e = ref.score(zin, tok)
    z64 = logits_f64(zin)
    want = logsumexp(z64, axis=1) - z64[np.arange(n), tok]
    np.testing.assert_allclose(e, want.astype(np.float32), rtol=2e-7, atol=0)
    ce = torch.nn.functional.cross_entropy(torch.from_numpy(z64), torch.from_numpy(tok).long(), reduction="none")
    np.testing.assert_allclose(e, ce.numpy().astype(np.float32), rtol=2e-7, atol=0)


def test_binary16_decoding_against_numpy(ref):
    # every binary16 bit pattern that is a number, as a one-column row: e = 0, and as the odd one out in a
    # two-column row against numpy's own float16 -> float64 conversion (subnormals, both zeros, extremes)
    bits = np.arange(0, 1 << 16, dtype=np.uint16)
    h = bits.view(np.float16)
    ok = np.isfinite(h)
    z = np.zeros((int(ok.sum()), 2), dtype=np.float16)
    z[:, 1] = h[ok]
    v = h[ok].astype(np.float64)
    e0 = ref.score(z, np.zeros(len(z), dtype=np.int32))
    np.testing.assert_allclose(e0, np.logaddexp(0.0, v).astype(np.float32), rtol=2e-7, atol=1e-12)      # log(1 + e^v)
    e1 = ref.score(z, np.ones(len(z), dtype=np.int32))
    np.testing.assert_allclose(e1, (np.logaddexp(0.0, v) - v).astype(np.float32), rtol=2e-7, atol=1e-12)


def test_token_id_selects_the_column_not_the_row(ref):
    # rows and columns carry different values: a transposed or mis-strided lookup fails here
    n, V = 5, 7
    z = (np.arange(n)[:, None] * 0.37 - np.arange(V)[None, :] * 0.91).astype(np.float32)
    tok = np.array([6, 0, 3, 1, 5], dtype=np.int32)
    e = ref.score(z, tok)
    z64 = z.astype(np.float64)
    want = np.array([math.log(np.exp(z64[r]).sum()) - z64[r, tok[r]] for r in range(n)])
    np.testing.assert_allclose(e, want.astype(np.float32), rtol=2e-7)


def test_shift_invariance_and_padding(ref):
    rng = np.random.default_rng(2)
    n, V, ld = 9, 1000, 1024
    z = np.full((n, ld), 1.0e4, dtype=np.float32)           # columns >= V are padding
    z[:, :V] = rng.standard_normal((n, V)) * 2
    tok = rng.integers(0, V, n).astype(np.int32)
    e = ref.score(z, tok, vocab=V)
    e_tight = ref.score(np.ascontiguousarray(z[:, :V]), tok)
    np.testing.assert_array_equal(e, e_tight)
    z2 = z.copy()
    z2[:, :V] += 16.0                                        # exact in binary32 for these magnitudes? no: compare loosely
    e2 = ref.score(z2, tok, vocab=V)
    np.testing.assert_allclose(e2, e, rtol=0, atol=2e-5)


def test_workload_generators_give_peaked_rows(ref):
    # the synthetic logits of the tiny workload: entropy scores are positive, finite and
    # the spiked rows whose token is the spiked id score lower than log V
    w = synth.WORKLOADS["tiny"]
    z = to_np(synth.make_logits(w, turn=1))
    tok = to_np(synth.make_token_ids(w, turn=1))
    e = ref.score(z, tok)
    assert np.isfinite(e).all() and (e > 0).all()
    z64 = z.astype(np.float64)
    want = logsumexp(z64, axis=1) - z64[np.arange(len(tok)), tok]
    np.testing.assert_allclose(e, want.astype(np.float32), rtol=2e-7)


def test_non_finite_cases(ref):
    V = 16
    z = np.zeros((5, V), dtype=np.float32)
    z[0, 3] = -np.inf                     # a -inf logit contributes nothing: log(V-1)
    z[1, 3] = -np.inf                     # ... and the token at it has probability 0: +inf
    z[2, :] = -np.inf                     # no finite maximum: NaN
    z[3, 5] = np.inf                      # +inf logit: NaN
    z[4, 7] = np.nan                      # NaN logit: NaN
    tok = np.array([0, 3, 0, 0, 0], dtype=np.int32)
    e = ref.score(z, tok)
    assert e[0] == np.float32(math.log(V - 1))
    assert e[1] == np.inf
    assert np.isnan(e[2]) and np.isnan(e[3]) and np.isnan(e[4])


def test_out_of_range_token_is_nan(ref):
    z = np.zeros((3, 10), dtype=np.float32)
    e = ref.score(z, np.array([-1, 10, 9], dtype=np.int32))
    assert np.isnan(e[0]) and np.isnan(e[1]) and e[2] == np.float32(math.log(10))


def test_empty_and_bad_arguments(ref):
    assert ref.score(np.zeros((0, 8), dtype=np.float32), np.zeros(0, dtype=np.int32)).shape == (0,)
    with pytest.raises(ValueError):
        ref.score(np.zeros((2, 8), dtype=np.float32), np.zeros(2, dtype=np.int32), vocab=9)
