"""Parity of sirllm_lmhead_score (token entropy straight from hidden states and the output embedding
matrix, paper Sec. 3.2) with the CPU oracle, through the C ABI, on one MI355X.

Tolerance: |gpu - ref| <= 2e-5 + 1e-5*|ref|.  The kernel's products of two bf16 / f16 numbers are exact in
binary32; a logit is their sum over d_model terms taken 16 at a time into a binary32 accumulator, i.e.
d_model/16 roundings, each off by at most 2^-24 * |partial sum| and by 2^-24 * |partial sum| / sqrt(3) in the root
mean square.  Adding like a random walk over the 256 roundings of d_model = 4096, with partial sums of order 10 on
these inputs, that is ~6e-6 per logit in the root mean square; the score is the token's logit minus a weighted mean
of logits (whose errors average out), plus the ~1e-6 of the softmax reduction.  Worst case seen over the 268
oracle-checked rows of the Llama-3-8B-shaped workload: 2.1e-5 (about three standard deviations), on scores of
5 to 15, where the bound is 7e-5 to 1.7e-4.  The relative term is the one the logits path uses.
"""
import numpy as np
import pytest
import torch

from helpers import to_np
from paper_2405_12528_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def b():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2405_12528_amd import binding
    return binding


def assert_close(gpu: np.ndarray, want: np.ndarray):
    nan_w, nan_g = np.isnan(want), np.isnan(gpu)
    np.testing.assert_array_equal(nan_g, nan_w)
    ok = ~nan_w
    err = np.abs(gpu[ok].astype(np.float64) - want[ok].astype(np.float64))
    tol = 2e-5 + 1e-5 * np.abs(want[ok].astype(np.float64))
    bad = err > tol
    assert not bad.any(), f"{bad.sum()} scores off; worst {err.max():.3e} (tolerance {tol[err.argmax()]:.3e})"
    return float(err.max()) if err.size else 0.0


def gpu_lmhead(b, h, w, tok, d_model=None, vocab=None):
    n = h.shape[0]
    V = w.shape[0] if vocab is None else vocab
    out = torch.full((n,), -12345.0, dtype=torch.float32, device=DEV)
    ws = torch.empty(max(b.sirllm_lmhead_workspace_bytes(n, V), 1), dtype=torch.uint8, device=DEV)
    b.sirllm_lmhead_score(h, w, tok, out, ws, d_model=d_model, vocab=vocab)
    torch.cuda.synchronize()
    return to_np(out)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("n_rows,d,V", [
    (64, 64, 1000),          # the tiny workload's shape: one token tile, four vocabulary tiles, ragged both ways
    (1, 8, 1),               # the smallest legal call
    (7, 72, 40),             # d_model not a multiple of the 64-wide pipeline stage
    (300, 512, 1000),        # two token tiles
    (513, 256, 777),         # three token tiles, the last one with a single row
    (257, 128, 2049),        # nine vocabulary tiles: the tile-to-XCD deal wraps, last tile has one column
    (5, 4096, 2500),         # the full inner dimension of the 7B / 8B shapes
    (256, 64, 256), (255, 64, 257),
])
def test_lmhead_score_matches_oracle(b, ref, dtype, n_rows, d, V):
    g = torch.Generator(device=DEV).manual_seed(n_rows * 7919 + V * 31 + d)
    h = (torch.randn((n_rows, d), generator=g, device=DEV) + 0.5).to(dtype)
    w = (torch.randn((V, d), generator=g, device=DEV) * (3.0 / d ** 0.5)).to(dtype)
    w[V // 2] += (4.0 / d)                                   # one token that many rows prefer
    tok = torch.randint(0, V, (n_rows,), generator=g, device=DEV, dtype=torch.int32)
    tok[::3] = V // 2
    got = gpu_lmhead(b, h, w, tok)
    want = ref.lmhead_score(to_np(h), to_np(w), to_np(tok))
    assert_close(got, want)


@pytest.mark.parametrize("n_rows,d,V", [
    (54, 4096, 32000),       # a turn of the Rock-Paper-Scissors-shaped dialogue: 128 x 64 tiles, W streamed once
    (1, 4096, 32000),        # one token (decode)
    (100, 1024, 5000),       # 65..128 rows: 128 x 128 tiles
    (128, 512, 1000), (65, 64, 129), (64, 32, 128),
    (33, 64, 70001),         # few rows, large vocabulary: 256 x 64 tiles, ragged last tile
    (20, 96, 66000),         # the same tiles with d_model a multiple of 32 only: stages of 32 K elements
    (128, 4096, 3000),       # 128 x 128 tiles over the full inner dimension, stages of 64 K elements
    (100, 128, 66000), (70, 96, 66000),   # 65..128 rows against a large vocabulary: 256 x 128 tiles, stages of 64 and of 32
    (200, 4096, 1500), (150, 96, 2000),   # 129..256 rows against a small vocabulary: 128 x 256 tiles, stages of 64 and of 32
    (300, 128, 66000), (384, 96, 66000),  # 257..384 rows against a large vocabulary: three token tiles of 256 x 128
])
def test_lmhead_few_rows_every_row_against_the_oracle(b, ref, n_rows, d, V):
    w_ = synth.WORKLOADS["rps_dialogue"]
    h, W = synth.make_lmhead(w_, turn=2, device=DEV, n_rows=n_rows, d_model=d, vocab=V)
    tok = torch.randint(0, V, (n_rows,), generator=torch.Generator(device=DEV).manual_seed(n_rows + V), device=DEV,
                        dtype=torch.int32)
    got = gpu_lmhead(b, h, W, tok)
    ref.set_threads(16)
    want = ref.lmhead_score(to_np(h), to_np(W), to_np(tok))
    assert_close(got, want)


def test_lmhead_random_shapes_and_paddings(b, ref):
    """Thirty random (rows, d_model, vocabulary) triples with random row paddings on both operands: every tile shape,
    both kernels (d_model a multiple of 32 or only of 8), ragged tiles on every side."""
    rng = np.random.default_rng(2405)
    ref.set_threads(16)
    for case in range(30):
        n = int(rng.choice([rng.integers(1, 65), rng.integers(65, 129), rng.integers(129, 700)]))
        d = 8 * int(rng.integers(1, 66))
        V = int(rng.integers(1, 3000))
        ld_h, ld_w = d + 8 * int(rng.integers(0, 4)), d + 8 * int(rng.integers(0, 4))
        dtype = (torch.bfloat16, torch.float16)[case % 2]
        g = torch.Generator(device=DEV).manual_seed(1000 + case)
        hbig = torch.full((n, ld_h), 300.0, device=DEV).to(dtype)                 # padding that would wreck the result
        wbig = torch.full((V + 3, ld_w), -300.0, device=DEV).to(dtype)
        hbig[:, :d] = (torch.randn((n, d), generator=g, device=DEV) + 0.5).to(dtype)
        wbig[:V, :d] = (torch.randn((V, d), generator=g, device=DEV) * (3.0 / d ** 0.5)).to(dtype)
        tok = torch.randint(0, V, (n,), generator=g, device=DEV, dtype=torch.int32)
        got = gpu_lmhead(b, hbig, wbig, tok, d_model=d, vocab=V)
        want = ref.lmhead_score(to_np(hbig), to_np(wbig), to_np(tok), d_model=d, vocab=V)
        try:
            assert_close(got, want)
        except AssertionError as e:
            raise AssertionError(f"case {case}: n={n} d={d} V={V} ld_h={ld_h} ld_w={ld_w} {dtype}: {e}") from None


def test_lmhead_leading_dimensions_and_subranges(b, ref):
    # hidden and weight embedded in larger allocations whose padding would wreck the result if it were read
    g = torch.Generator(device=DEV).manual_seed(5)
    n, d, V = 70, 200, 900
    hbig = torch.full((n, 256), 1.0e3, device=DEV).to(torch.bfloat16)
    wbig = torch.full((V + 50, 320), -1.0e3, device=DEV).to(torch.bfloat16)
    hbig[:, :d] = torch.randn((n, d), generator=g, device=DEV).to(torch.bfloat16)
    wbig[:V, :d] = (torch.randn((V, d), generator=g, device=DEV) * 0.2).to(torch.bfloat16)
    tok = torch.randint(0, V, (n,), generator=g, device=DEV, dtype=torch.int32)
    got = gpu_lmhead(b, hbig, wbig, tok, d_model=d, vocab=V)
    want = ref.lmhead_score(to_np(hbig), to_np(wbig), to_np(tok), d_model=d, vocab=V)
    assert_close(got, want)
    tight = ref.lmhead_score(np.ascontiguousarray(to_np(hbig)[:, :d]), np.ascontiguousarray(to_np(wbig)[:V, :d]), to_np(tok))
    np.testing.assert_array_equal(want, tight)


def test_lmhead_out_of_range_token_is_nan(b, ref):
    g = torch.Generator(device=DEV).manual_seed(6)
    n, d, V = 6, 64, 300
    h = torch.randn((n, d), generator=g, device=DEV).to(torch.bfloat16)
    w = torch.randn((V, d), generator=g, device=DEV).to(torch.bfloat16)
    tok = torch.tensor([0, -1, V, V - 1, 2 ** 31 - 1, 17], dtype=torch.int32, device=DEV)
    got = gpu_lmhead(b, h, w, tok)
    want = ref.lmhead_score(to_np(h), to_np(w), to_np(tok))
    assert np.isnan(want[[1, 2, 4]]).all()
    assert_close(got, want)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("n,d,V", [(6, 64, 300), (70, 96, 700), (300, 72, 600)])    # fast and general kernels, all tile shapes
def test_lmhead_non_finite_operands(b, ref, dtype, n, d, V):
    """Non-finite logits behave as in the logits path: a -inf logit adds nothing, a token at a -inf logit scores
    +inf, a row with a NaN or a +inf logit scores NaN."""
    g = torch.Generator(device=DEV).manual_seed(n + d)
    h = (torch.rand((n, d), generator=g, device=DEV) + 0.5).to(dtype)          # all positive
    w = torch.randn((V, d), generator=g, device=DEV).to(dtype)
    w[7, 3] = float("-inf")                                                   # logit 7 is -inf for every row ...
    w[V - 1, d - 1] = float("-inf")                                           # ... and so is the last one
    h[1, 5] = float("nan")                                                    # row 1: every logit NaN
    h[3, 9] = float("inf")                                                    # row 3: +inf and -inf logits, NaN where both meet
    tok = torch.randint(0, V, (n,), generator=g, device=DEV, dtype=torch.int32)
    tok[2] = 7                                                                # row 2's own token sits at a -inf logit
    tok[4] = V - 1
    got = gpu_lmhead(b, h, w, tok)
    want = ref.lmhead_score(to_np(h), to_np(w), to_np(tok))
    assert np.isnan(want[1]) and np.isnan(want[3]) and np.isposinf(want[2]) and np.isposinf(want[4])
    assert np.isfinite(want[[0, 5]]).all()
    inf_w = np.isinf(want)
    np.testing.assert_array_equal(np.isinf(got), inf_w)
    np.testing.assert_array_equal(got[inf_w], want[inf_w])
    assert_close(np.where(inf_w, 0, got), np.where(inf_w, 0, want))


def test_lmhead_closed_forms(b):
    # equal output embeddings -> log V for every row; a zero hidden state -> log V
    V, d = 1000, 64
    h = torch.randn((3, d), device=DEV).to(torch.bfloat16)
    h[2] = 0
    w = torch.randn((1, d), device=DEV).to(torch.bfloat16).repeat(V, 1).contiguous()
    tok = torch.tensor([0, 500, 999], dtype=torch.int32, device=DEV)
    got = gpu_lmhead(b, h, w, tok)
    np.testing.assert_allclose(got, np.float32(np.log(V)), rtol=0, atol=2e-6)


def test_lmhead_agrees_with_scoring_the_materialised_logits(b):
    # the same quantity by the other route: logits written out in binary32, then the logits scan
    w_ = synth.WORKLOADS["llama2_7b"]
    n, V = 300, 32000
    h, W = synth.make_lmhead(w_, turn=1, device=DEV, n_rows=n)
    tok = synth.make_token_ids(w_, turn=1, device=DEV, n_rows=n)
    got = gpu_lmhead(b, h, W, tok)
    z = h.float() @ W.float().T
    out = torch.empty(n, device=DEV)
    b.sirllm_score(z, tok, out)
    torch.cuda.synchronize()
    assert_close(got, to_np(out))


@pytest.mark.timeout(600)
def test_lmhead_llama3_shape_a_whole_token_tile_against_the_oracle(b, ref):
    """2048 x 4096 hidden states against a 128256 x 4096 output embedding (the Llama-3-8B-shaped workload): one whole
    256-row token tile (rows 256..511: every lane, wave and accumulator block of a workgroup, against all 501
    vocabulary tiles) and 12 rows sampled from the other tiles are checked against the oracle's double-precision
    product; every row is also checked against the logits route."""
    w_ = synth.WORKLOADS["llama3_8b"]
    h, W = synth.make_lmhead(w_, turn=1, device=DEV)
    tok = synth.make_token_ids(w_, turn=1, device=DEV)
    n = h.shape[0]
    assert (n, W.shape[0], W.shape[1]) == (2048, 128256, 4096)
    got = gpu_lmhead(b, h, W, tok)
    assert np.isfinite(got).all() and (got > 0).all()
    # every row, against the logits scan fed with binary32 products (256 rows at a time: 131 MB of logits)
    other = torch.empty(n, device=DEV)
    Wf = W.float()
    for r0 in range(0, n, 256):
        z = h[r0:r0 + 256].float() @ Wf.T
        b.sirllm_score(z, tok[r0:r0 + 256], other[r0:r0 + 256])
    torch.cuda.synchronize()
    assert_close(got, to_np(other))
    rows = np.concatenate([np.arange(256, 512), np.random.default_rng(0).choice(np.r_[0:256, 512:n], 12, replace=False)])
    rows.sort()
    ref.set_threads(16)
    want = ref.lmhead_score(to_np(h[torch.from_numpy(rows).to(DEV)]), to_np(W), to_np(tok)[rows])
    worst = assert_close(got[rows], want)
    print(f"llama3 shape: worst |gpu - oracle| over {len(rows)} rows (one whole token tile + 12 sampled) = {worst:.2e}")


# ------------------------------------------------------------------ the whole step, scores from the LM head
def gpu_step_lmhead(b, pol, h, W, tok, held, k_c, v_c):
    n_streams, n_held = held.shape
    n_new = h.shape[0] // n_streams
    n_cand = n_held + n_new
    n_keep = min(n_cand, pol.n_sink + pol.n_topk + pol.n_recent)
    E = torch.full((n_streams, n_cand), -5.0, device=DEV)
    E[:, :n_held] = held
    idx = torch.full((n_streams, max(n_keep, 1)), -7, dtype=torch.int32, device=DEV)
    out = torch.full((n_streams, max(n_keep, 1)), -7.0, device=DEV)
    shape = k_c.shape[:3] + (n_keep,) + k_c.shape[4:]
    k_dst = torch.zeros(shape, dtype=k_c.dtype, device=DEV)
    v_dst = torch.zeros(shape, dtype=v_c.dtype, device=DEV)
    ws = torch.empty(max(b.sirllm_step_lmhead_workspace_bytes(n_streams, n_cand, h.shape[0], W.shape[0]), 256),
                     dtype=torch.uint8, device=DEV)
    got = b.sirllm_step_lmhead(h, W, tok, E, n_held, n_new, pol, k_c, v_c, k_dst, v_dst, idx, out, ws)
    torch.cuda.synchronize()
    assert got == n_keep
    return dict(E=E, idx=idx[:, :n_keep], out=out[:, :n_keep], k=k_dst, v=v_dst, n_keep=n_keep, evicted=n_cand > n_keep)


def check_step_lmhead(ref, pol, h, W, tok, held, k_c, v_c, g):
    """New scores against the oracle's double-precision product; then the oracle's select + gather, fed the GPU's
    scores, bit for bit."""
    n_streams, n_held = held.shape
    n_new = h.shape[0] // n_streams
    Eg = to_np(g["E"])
    if n_new:
        want = ref.lmhead_score(to_np(h), to_np(W), to_np(tok)).reshape(n_streams, n_new)
        assert_close(Eg[:, n_held:].reshape(-1), want.reshape(-1))
    np.testing.assert_array_equal(Eg[:, :n_held].view(np.uint32), to_np(held).view(np.uint32))
    ri, ro = ref.decay_select(Eg, n_held, n_new, ref.Policy(*pol))
    np.testing.assert_array_equal(to_np(g["idx"]), ri)
    np.testing.assert_array_equal(to_np(g["out"]).view(np.uint32), ro.view(np.uint32))
    if g["evicted"]:
        rk, rv = ref.compact_kv(to_np(k_c), to_np(v_c), ri, n_src=n_held + n_new)
        assert np.array_equal(to_np(g["k"]), rk) and np.array_equal(to_np(g["v"]), rv)
    else:
        assert not to_np(g["k"]).any() and not to_np(g["v"]).any()


@pytest.mark.parametrize("n_streams,n_held,n_new,pol,d,V", [
    (1, 100, 40, (4, 50, 40, 0.9), 64, 777),     # new tokens all inside the recent window
    (1, 100, 40, (4, 80, 8, 0.9), 64, 777),      # selection depends on this turn's scores
    (3, 60, 30, (4, 30, 10, 0.8), 128, 1000),    # several streams: rows of one launch go to different score rows
    (2, 10, 12, (4, 20, 8, 0.9), 72, 300),       # under budget; d_model on the general kernel
    (2, 90, 0, (4, 20, 8, 0.9), 64, 300),        # no new tokens
    (1, 0, 50, (4, 20, 8, 0.9), 64, 300),        # empty cache
    (2, 33000, 100, (4, 30000, 200, 0.9), 64, 300),   # above 32768 slots: the selection's scratch sits behind the LM head's
])
def test_step_lmhead_small_shapes(b, ref, n_streams, n_held, n_new, pol, d, V):
    pol = b.Policy(*pol)
    g0 = torch.Generator(device=DEV).manual_seed(n_held * 100 + n_new + d)
    h = torch.randn((n_streams * n_new, d), generator=g0, device=DEV).to(torch.bfloat16)
    W = (torch.randn((V, d), generator=g0, device=DEV) * (3.0 / d ** 0.5)).to(torch.bfloat16)
    tok = torch.randint(0, V, (n_streams * n_new,), generator=g0, device=DEV, dtype=torch.int32)
    held = torch.rand((n_streams, n_held), generator=g0, device=DEV) * 6
    k_c = torch.randn((n_streams, 2, 2, n_held + n_new, 16), generator=g0, device=DEV)
    v_c = torch.randn((n_streams, 2, 2, n_held + n_new, 16), generator=g0, device=DEV)
    g = gpu_step_lmhead(b, pol, h, W, tok, held, k_c, v_c)
    check_step_lmhead(ref, pol, h, W, tok, held, k_c, v_c, g)


def test_cache_step_from_hidden_four_turns(b, ref):
    """The tiny workload through RetentiveCache.step_from_hidden: 64 tokens per turn, budget 32, the output
    embedding fixed across turns, every turn checked against the oracle fed the GPU's scores."""
    from paper_2405_12528_amd.cache import RetentiveCache
    w = synth.WORKLOADS["tiny"]
    pol = b.Policy(w.n_sink, w.n_topk, w.n_recent, w.decay)
    cache = RetentiveCache(1, w.n_layers, w.n_kv_heads, w.head_dim, pol, max_new=w.n_new, kv_dtype=torch.float32, device=DEV)
    for turn in range(1, w.n_turns + 1):
        h, W = synth.make_lmhead(w, turn=turn, device=DEV)
        tok = synth.make_token_ids(w, turn=turn, device=DEV)
        kn, vn = cache.new_kv_slots(w.n_new)
        kn.copy_(synth.make_kv(w, n_pos=w.n_new, turn=turn, device=DEV, which="k"))
        vn.copy_(synth.make_kv(w, n_pos=w.n_new, turn=turn, device=DEV, which="v"))
        n_held = cache.n_held
        held = cache.scores[:, :n_held].clone()
        k_c = cache.k[:, :, :, :n_held + w.n_new].clone()
        v_c = cache.v[:, :, :, :n_held + w.n_new].clone()
        evicted = cache.step_from_hidden(h, W, tok)
        torch.cuda.synchronize()
        assert evicted and cache.n_held == w.budget
        # what the step appended behind the held scores is no longer reachable through the cache object: score again
        new = torch.empty(w.n_new, device=DEV)
        ws = torch.empty(b.sirllm_lmhead_workspace_bytes(w.n_new, w.vocab), dtype=torch.uint8, device=DEV)
        b.sirllm_lmhead_score(h, W, tok, new, ws)
        torch.cuda.synchronize()
        want = ref.lmhead_score(to_np(h), to_np(W), to_np(tok))
        assert_close(to_np(new), want)
        Eg = np.concatenate([to_np(held), to_np(new)[None, :]], axis=1)
        ri, ro = ref.decay_select(Eg, n_held, w.n_new, ref.Policy(*pol))
        np.testing.assert_array_equal(to_np(cache.kept_idx[:, :w.budget]), ri)
        np.testing.assert_array_equal(to_np(cache.scores[:, :w.budget]).view(np.uint32), ro.view(np.uint32))
        rk, rv = ref.compact_kv(to_np(k_c), to_np(v_c), ri)
        assert np.array_equal(to_np(cache.k[:, :, :, :w.budget]), rk) and np.array_equal(to_np(cache.v[:, :, :, :w.budget]), rv)


def test_step_lmhead_mistral_shape(b, ref):
    """Mistral-7B-shaped step (1024 new tokens, V = 32000, d_model 4096, budget 4096 of 8192 candidates, K/V 32 x 8 x
    128 bf16) with the scores from the LM head: every score against the logits route, 8 sampled rows against the
    oracle's product, selection and K/V against the oracle fed the GPU's scores."""
    w = synth.WORKLOADS["mistral_7b"]
    pol = b.Policy(w.n_sink, w.n_topk, w.n_recent, w.decay)
    h, W = synth.make_lmhead(w, turn=1, device=DEV)
    tok = synth.make_token_ids(w, turn=1, device=DEV)
    held = synth.make_held_scores(w, device=DEV)
    k_c = synth.make_kv(w, device=DEV, which="k")
    v_c = synth.make_kv(w, device=DEV, which="v")
    g = gpu_step_lmhead(b, pol, h, W, tok, held, k_c, v_c)
    Eg = to_np(g["E"])
    z = h.float() @ W.float().T
    other = torch.empty(w.n_new, device=DEV)
    b.sirllm_score(z, tok, other)
    torch.cuda.synchronize()
    assert_close(Eg[0, w.n_held:], to_np(other))
    rows = np.sort(np.random.default_rng(1).choice(w.n_new, 8, replace=False))
    ref.set_threads(16)
    want = ref.lmhead_score(to_np(h[torch.from_numpy(rows).to(DEV)]), to_np(W), to_np(tok)[rows])
    assert_close(Eg[0, w.n_held:][rows], want)
    ri, ro = ref.decay_select(Eg, w.n_held, w.n_new, ref.Policy(*pol))
    np.testing.assert_array_equal(to_np(g["idx"]), ri)
    np.testing.assert_array_equal(to_np(g["out"]).view(np.uint32), ro.view(np.uint32))
    rk, rv = ref.compact_kv(to_np(k_c), to_np(v_c), ri)
    assert np.array_equal(to_np(g["k"]), rk) and np.array_equal(to_np(g["v"]), rv)


def test_step_lmhead_replays_from_a_captured_graph(b):
    """sirllm_step_lmhead allocates nothing and synchronises nothing; its kernels ask for more than 64 KB of dynamic
    LDS (a function attribute set at launch).  Captured into a HIP graph, every replay must reproduce the eager
    result, also with eager work and synchronisations between replays."""
    pol = b.Policy(4, 30, 0, 0.8)
    S, n_held, n_new, V, d = 2, 60, 40, 777, 128
    g0 = torch.Generator(device=DEV).manual_seed(5)
    h = torch.randn((S * n_new, d), generator=g0, device=DEV).to(torch.bfloat16)
    W = (torch.randn((V, d), generator=g0, device=DEV) * 0.3).to(torch.bfloat16)
    tok = torch.randint(0, V, (S * n_new,), generator=g0, device=DEV, dtype=torch.int32)
    held = torch.rand((S, n_held), generator=g0, device=DEV) * 6
    k_c = torch.randn((S, 2, 2, n_held + n_new, 16), generator=g0, device=DEV)
    v_c = torch.randn((S, 2, 2, n_held + n_new, 16), generator=g0, device=DEV)
    n_keep = 34
    ws = torch.empty(b.sirllm_step_lmhead_workspace_bytes(S, n_held + n_new, S * n_new, V), dtype=torch.uint8, device=DEV)

    def fresh():
        E = torch.zeros((S, n_held + n_new), device=DEV)
        E[:, :n_held] = held
        return dict(E=E, idx=torch.zeros((S, n_keep), dtype=torch.int32, device=DEV),
                    out=torch.zeros((S, n_keep), device=DEV), k=torch.zeros((S, 2, 2, n_keep, 16), device=DEV),
                    v=torch.zeros((S, 2, 2, n_keep, 16), device=DEV))

    def run(t):
        b.sirllm_step_lmhead(h, W, tok, t["E"], n_held, n_new, pol, k_c, v_c, t["k"], t["v"], t["idx"], t["out"], ws)

    eager = fresh()
    run(eager)
    torch.cuda.synchronize()
    cap = fresh()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(cap)                                         # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(cap)
    for rep in range(4):
        for name, t in cap.items():                      # eager work between replays: wipe every output
            t.zero_() if name != "E" else t[:, n_held:].zero_()
        ws.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name in eager:
            assert torch.equal(cap[name], eager[name]), f"replay {rep}: {name} differs from the eager run"


def test_lmhead_score_is_deterministic(b):
    # no atomics, fixed summation order per tile shape: the same call gives the same bytes
    g = torch.Generator(device=DEV).manual_seed(9)
    for n, d, V in ((300, 512, 5000), (54, 1024, 3000), (100, 256, 2000)):
        h = torch.randn((n, d), generator=g, device=DEV).to(torch.bfloat16)
        W = (torch.randn((V, d), generator=g, device=DEV) * 0.2).to(torch.bfloat16)
        tok = torch.randint(0, V, (n,), generator=g, device=DEV, dtype=torch.int32)
        first = gpu_lmhead(b, h, W, tok)
        for _ in range(10):
            np.testing.assert_array_equal(gpu_lmhead(b, h, W, tok).view(np.uint32), first.view(np.uint32))
