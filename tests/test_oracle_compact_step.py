"""Pins for the oracle's KV compaction and whole step (paper Sec. 3.3, Algorithm 1): numpy
fancy indexing as the library routine, self-identifying payloads, strided layouts, and the
multi-turn invariants of the tiny workload.  CPU only."""
import numpy as np
import pytest
from scipy.special import logsumexp

from helpers import to_np
from paper_2405_12528_amd import synth


def test_gather_equals_numpy_indexing_on_tagged_payload(ref):
    S, L, H, Pn, D = 2, 3, 2, 17, 8
    k = to_np(synth.tagged_kv(S, L, H, Pn, D, which=0))
    v = to_np(synth.tagged_kv(S, L, H, Pn, D, which=1))
    kept = np.array([[0, 1, 4, 9, 15, 16], [2, 3, 5, 7, 11, 13]], dtype=np.int32)
    kd, vd = ref.compact_kv(k, v, kept)
    for s in range(S):
        np.testing.assert_array_equal(kd[s], k[s][:, :, kept[s], :])
        np.testing.assert_array_equal(vd[s], v[s][:, :, kept[s], :])
    # every element still names its source coordinates
    assert kd[1, 2, 1, 3, 5] == k[1, 2, 1, 7, 5]
    assert (vd != kd).all()


@pytest.mark.parametrize("dtype", [np.uint8, np.uint16, np.float32, np.float64])
def test_gather_is_a_byte_copy_for_every_element_size(ref, dtype):
    rng = np.random.default_rng(0)
    k = rng.integers(0, 255, (1, 2, 2, 9, 4)).astype(dtype)
    kept = np.array([[8, 0, 3]], dtype=np.int32)               # any order the caller gives is honoured
    kd, _ = ref.compact_kv(k, None, kept)
    np.testing.assert_array_equal(kd[0], k[0][:, :, [8, 0, 3], :])


def test_gather_through_strided_source(ref):
    # source cache embedded in a larger allocation: slots padded, heads padded
    big = np.arange(1 * 2 * 3 * 20 * 12, dtype=np.int32).reshape(1, 2, 3, 20, 12)
    src = big[:, :, :2, :15, :8]                                # non-contiguous view, last axis contiguous
    kept = np.array([[1, 2, 14]], dtype=np.int32)
    kd, _ = ref.compact_kv(src, None, kept)
    np.testing.assert_array_equal(kd[0], src[0][:, :, [1, 2, 14], :])


def test_out_of_range_index_gives_zero_row(ref):
    k = np.ones((1, 1, 1, 4, 4), dtype=np.float32)
    kd, _ = ref.compact_kv(k, None, np.array([[0, 4, -1, 3]], dtype=np.int32))
    assert kd[0, 0, 0].tolist() == [[1] * 4, [0] * 4, [0] * 4, [1] * 4]
    kd, _ = ref.compact_kv(k, None, np.array([[0, 3]], dtype=np.int32), n_src=3)
    assert kd[0, 0, 0].tolist() == [[1] * 4, [0] * 4]


def test_step_is_score_then_decay_select_then_gather(ref):
    w = synth.WORKLOADS["tiny"]
    pol = ref.Policy(w.n_sink, w.n_topk, w.n_recent, w.decay)
    rng = np.random.default_rng(4)
    n_held, n_new = 32, w.n_new
    z = to_np(synth.make_logits(w, turn=2))
    tok = to_np(synth.make_token_ids(w, turn=2))
    held = rng.gamma(2.0, 2.0, (1, n_held)).astype(np.float32)
    k = to_np(synth.make_kv(w, n_pos=n_held + n_new, which="k"))
    v = to_np(synth.make_kv(w, n_pos=n_held + n_new, which="v"))
    r = ref.step(z, tok, w.vocab, held, n_new, pol, k, v)
    # scores: float64 library routine
    z64 = z.astype(np.float64)
    want_e = (logsumexp(z64, axis=1) - z64[np.arange(n_new), tok]).astype(np.float32)
    np.testing.assert_allclose(r["new_scores"][0], want_e, rtol=2e-7)
    # selection: the separate entry point on the appended array
    cand = np.concatenate([held, r["new_scores"]], axis=1)
    kept, out = ref.decay_select(cand, n_held, n_new, pol)
    np.testing.assert_array_equal(r["kept_idx"], kept)
    np.testing.assert_array_equal(r["scores_out"], out)
    assert r["evicted"] and kept.shape[1] == w.budget
    # new scores enter undecayed, held ones decayed once
    for j, i in enumerate(kept[0]):
        want = cand[0, i] if i >= n_held else np.float32(cand[0, i] * np.float32(w.decay))
        assert r["scores_out"][0, j] == want
    np.testing.assert_array_equal(r["k"][0], k[0][:, :, kept[0], :])
    np.testing.assert_array_equal(r["v"][0], v[0][:, :, kept[0], :])


def test_tiny_dialogue_four_turns(ref):
    """The tiny workload end to end: 64 new tokens per turn over 4 turns, budget 32."""
    w = synth.WORKLOADS["tiny"]
    pol = ref.Policy(w.n_sink, w.n_topk, w.n_recent, w.decay)
    E = np.zeros((1, 0), dtype=np.float32)
    shape0 = (1, w.n_layers, w.n_kv_heads, 0, w.head_dim)
    K, V = np.zeros(shape0, np.float32), np.zeros(shape0, np.float32)
    origin = np.zeros((0, 2), dtype=int)                        # (turn, token) of every cached slot
    first_scores = {}
    for turn in range(1, w.n_turns + 1):
        z = to_np(synth.make_logits(w, turn=turn))
        tok = to_np(synth.make_token_ids(w, turn=turn))
        k_new = to_np(synth.make_kv(w, n_pos=w.n_new, turn=turn, which="k"))
        v_new = to_np(synth.make_kv(w, n_pos=w.n_new, turn=turn, which="v"))
        K_c = np.concatenate([K, k_new], axis=3)
        V_c = np.concatenate([V, v_new], axis=3)
        org_c = np.concatenate([origin, np.stack([np.full(w.n_new, turn), np.arange(w.n_new)], axis=1)])
        n_held = E.shape[1]
        assert n_held + w.n_new == (64 if turn == 1 else 96)
        r = ref.step(z, tok, w.vocab, E, w.n_new, pol, K_c, V_c)
        kept = r["kept_idx"][0]
        for t in range(w.n_new):
            first_scores[(turn, t)] = r["new_scores"][0, t]
        # budget, sinks, recent window
        assert len(kept) == w.budget
        assert kept[:w.n_sink].tolist() == [0, 1, 2, 3]
        assert kept[-w.n_recent:].tolist() == list(range(n_held + w.n_new - w.n_recent, n_held + w.n_new))
        origin = org_c[kept]
        E, K, V = r["scores_out"], r["k"], r["v"]
        # the sinks are the first four tokens of the dialogue for ever
        assert origin[:4].tolist() == [[1, 0], [1, 1], [1, 2], [1, 3]]
        # every cached score is its first score decayed once per turn since (binary32 product)
        for j, (t0, i0) in enumerate(origin):
            want = first_scores[(t0, i0)]
            for _ in range(turn - t0):
                want = np.float32(want * np.float32(w.decay))
            assert E[0, j] == want
        # K/V rows travel with their tokens
        for j, (t0, i0) in enumerate(origin):
            src = to_np(synth.make_kv(w, n_pos=w.n_new, turn=int(t0), which="k"))
            np.testing.assert_array_equal(K[0, :, :, j, :], src[0, :, :, i0, :])
    assert E.shape == (1, w.budget)


def test_inplace_gather_equals_out_of_place_and_leaves_the_tail(ref):
    rng = np.random.default_rng(8)
    S, L, H, Pn, D = 2, 2, 3, 40, 8
    k = to_np(synth.tagged_kv(S, L, H, Pn, D, which=0))
    v = to_np(synth.tagged_kv(S, L, H, Pn, D, which=1))
    kept = np.stack([np.sort(rng.choice(Pn, 17, replace=False)) for _ in range(S)]).astype(np.int32)
    kept[0, :5] = [0, 1, 2, 3, 4]                              # a leading run that does not move
    want_k = np.stack([k[s][:, :, kept[s], :] for s in range(S)])     # numpy fancy indexing on the old content
    want_v = np.stack([v[s][:, :, kept[s], :] for s in range(S)])
    k2, v2 = k.copy(), v.copy()
    ref.compact_kv_inplace(k2, v2, kept)
    np.testing.assert_array_equal(k2[:, :, :, :17], want_k)
    np.testing.assert_array_equal(v2[:, :, :, :17], want_v)
    np.testing.assert_array_equal(k2[:, :, :, 17:], k[:, :, :, 17:])  # slots past n_keep untouched
    kd, vd = ref.compact_kv(k, v, kept)
    np.testing.assert_array_equal(k2[:, :, :, :17], kd)
    # a chain where every row is the source of its left neighbour: needs the old content throughout
    chain = np.arange(1, 31, dtype=np.int32)[None, :].repeat(S, 0)
    k3 = k.copy()
    ref.compact_kv_inplace(k3, None, chain)
    np.testing.assert_array_equal(k3[:, :, :, :30], k[:, :, :, 1:31])


def test_ragged_step_is_the_uniform_step_stream_by_stream(ref):
    # every stream of a ragged batch must come out exactly as if it had been stepped alone
    rng = np.random.default_rng(3)
    pol = ref.Policy(4, 20, 8, 0.9)
    V, S, L, H, D = 300, 4, 2, 2, 8
    n_held, n_new = [0, 40, 10, 90], [12, 30, 0, 7]
    cap = max(h + n for h, n in zip(n_held, n_new))
    z = (rng.standard_normal((sum(n_new), V)) * 2).astype(np.float32)
    tok = rng.integers(0, V, sum(n_new)).astype(np.int32)
    scores = np.full((S, cap), np.nan, dtype=np.float32)
    for s in range(S):
        scores[s, :n_held[s]] = rng.gamma(2.0, 2.0, n_held[s])
    k = rng.standard_normal((S, L, H, cap, D)).astype(np.float32)
    v = rng.standard_normal((S, L, H, cap, D)).astype(np.float32)
    k0, v0, s0 = k.copy(), v.copy(), scores.copy()
    kept, out, keep_n = ref.step_ragged(z, tok, V, scores, n_held, n_new, pol, k, v)
    r0 = 0
    for s in range(S):
        h, n = n_held[s], n_new[s]
        alone = ref.step(np.ascontiguousarray(z[r0:r0 + n]).reshape(n, V), tok[r0:r0 + n], V, s0[s:s + 1, :h], n, pol,
                         np.ascontiguousarray(k0[s:s + 1, :, :, :h + n]), np.ascontiguousarray(v0[s:s + 1, :, :, :h + n]))
        r0 += n
        np.testing.assert_array_equal(kept[s], alone["kept_idx"][0])
        np.testing.assert_array_equal(out[s], alone["scores_out"][0])
        np.testing.assert_array_equal(scores[s, h:h + n], alone["new_scores"][0])
        assert keep_n[s] == min(h + n, 32)
        np.testing.assert_array_equal(k[s, :, :, :keep_n[s]], alone["k"][0])
        np.testing.assert_array_equal(v[s, :, :, :keep_n[s]], alone["v"][0])
        if h + n <= 32:
            np.testing.assert_array_equal(k[s], k0[s])          # nothing evicted: cache untouched
