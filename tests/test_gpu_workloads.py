"""Parity at the full sizes of the benchmark workloads, in the launch configuration bench.py
times (sirllm_step on the default launch shapes), against the CPU oracle on the same bytes.

Scores: every row, |gpu - ref| <= 1e-6 + 1e-5*|ref|.  Kept indices and compacted scores: every
stream, bit exact, oracle fed the GPU's scores.  K/V: bit exact, the whole tensors for the
single-stream workloads and, one stream at a time from the pre-step buffers, for every stream of
the 32-stream dialogue at its checked turns."""
import os

import numpy as np
import pytest
import torch

from helpers import to_np
from paper_2405_12528_amd import synth
from test_gpu_parity import assert_scores_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def b():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2405_12528_amd import binding
    return binding


@pytest.mark.timeout(300)
@pytest.mark.parametrize("name", ["llama2_7b", "mistral_7b", "llama3_8b", "llama3_8k_budget"])
def test_full_size_step(b, ref, name):
    w = synth.WORKLOADS[name]
    ref.set_threads(16)
    pol = b.Policy(w.n_sink, w.n_topk, w.n_recent, w.decay)
    S, n_held, n_new, n_cand, n_keep = w.n_streams, w.n_held, w.n_new, w.n_cand, w.n_keep
    logits = synth.make_logits(w, turn=1, device=DEV)
    tok = synth.make_token_ids(w, turn=1, device=DEV)
    scores = torch.full((S, n_cand), -3.0, device=DEV)
    held = synth.make_held_scores(w, device=DEV)
    scores[:, :n_held] = held
    k_src = synth.make_kv(w, device=DEV, which="k")
    v_src = synth.make_kv(w, device=DEV, which="v")
    dst_shape = (S, w.n_layers, w.n_kv_heads, n_keep, w.head_dim)
    k_dst = torch.zeros(dst_shape, dtype=k_src.dtype, device=DEV)
    v_dst = torch.zeros(dst_shape, dtype=k_src.dtype, device=DEV)
    kept = torch.full((S, n_keep), -1, dtype=torch.int32, device=DEV)
    out = torch.full((S, n_keep), -1.0, device=DEV)
    assert b.sirllm_step(logits, tok, w.vocab, scores, n_held, n_new, pol, k_src, v_src, k_dst, v_dst, kept, out) == n_keep
    torch.cuda.synchronize()

    Eg = to_np(scores)
    want = ref.score(to_np(logits), to_np(tok), vocab=w.vocab).reshape(S, n_new)
    assert_scores_close(Eg[:, n_held:], want)
    np.testing.assert_array_equal(Eg[:, :n_held].view(np.uint32), to_np(held).view(np.uint32))
    ri, ro = ref.decay_select(Eg, n_held, n_new, ref.Policy(*pol))
    np.testing.assert_array_equal(to_np(kept), ri)
    np.testing.assert_array_equal(to_np(out).view(np.uint32), ro.view(np.uint32))
    # invariants of the policy (paper Sec. 3.1, 3.3)
    assert ri.shape[1] == w.budget and (np.diff(ri, axis=1) > 0).all()
    assert ri[0, :w.n_sink].tolist() == list(range(w.n_sink))
    assert ri[0, -w.n_recent:].tolist() == list(range(n_cand - w.n_recent, n_cand))
    rk, rv = ref.compact_kv(to_np(k_src), to_np(v_src), ri, n_src=n_cand)
    assert np.array_equal(to_np(k_dst), rk), "compacted K differs from the oracle"
    assert np.array_equal(to_np(v_dst), rv), "compacted V differs from the oracle"


@pytest.mark.timeout(300)
@pytest.mark.parametrize("name,held_new", [
    ("llama3_8b", None),                                                         # the shape bench.py times, through the ragged calls
    ("mistral_7b", None),
    ("batched_dialogue", [(2048, 256), (1500, 256), (2048, 100), (300, 256)]),   # unequal streams of the dialogue shape
])
def test_full_size_ragged_two_buffer_step(b, ref, name, held_new):
    """sirllm_step_ragged_out_of_place at the benchmark shapes (the launch bench.py times as the ragged out-of-place step): scores,
    kept lists, compacted scores and the whole destination K/V of every stream against the oracle; the source is not written."""
    w = synth.WORKLOADS[name]
    ref.set_threads(16)
    pol = b.Policy(w.n_sink, w.n_topk, w.n_recent, w.decay)
    if held_new is None:
        held_new = [(w.n_held, w.n_new)] * w.n_streams
    S = len(held_new)
    n_held = np.array([h for h, _ in held_new]); n_new = np.array([n for _, n in held_new])
    n_cand = n_held + n_new
    max_cand, total, budget = int(n_cand.max()), int(n_new.sum()), w.budget
    g0 = torch.Generator(device=DEV).manual_seed(5)
    dt = torch.float32 if w.logits_dtype == "f32" else torch.bfloat16
    z = (torch.randn((total, w.vocab), generator=g0, device=DEV) * w.sigma).to(dt)
    tok = torch.randint(0, w.vocab, (total,), generator=g0, device=DEV, dtype=torch.int32)
    scores = torch.full((S, max_cand), -3.0, device=DEV)
    for s in range(S):
        scores[s, :n_held[s]] = torch.rand((int(n_held[s]),), generator=g0, device=DEV) * 9.0
    shape = (S, w.n_layers, w.n_kv_heads, max_cand, w.head_dim)
    k = torch.randint(-30000, 30000, shape, generator=g0, device=DEV, dtype=torch.int16).view(torch.bfloat16)
    v = torch.randint(-30000, 30000, shape, generator=g0, device=DEV, dtype=torch.int16).view(torch.bfloat16)
    keep_cap = min(max_cand, budget)
    kd = torch.full((S, w.n_layers, w.n_kv_heads, keep_cap, w.head_dim), 77, dtype=torch.bfloat16, device=DEV)
    vd = torch.full_like(kd, 77)
    kept = torch.full((S, keep_cap), -7, dtype=torch.int32, device=DEV)
    out = torch.full((S, keep_cap), -7.0, device=DEV)
    n_keep_dev = torch.full((S,), -9, dtype=torch.int32, device=DEV)
    held_dev = torch.from_numpy(n_held.astype(np.int32)).to(DEV)
    cu = torch.from_numpy(np.concatenate([[0], np.cumsum(n_new)]).astype(np.int32)).to(DEV)
    hs = to_np(scores).copy()
    k_sum, v_sum = k.view(torch.int16).sum(dtype=torch.int64).item(), v.view(torch.int16).sum(dtype=torch.int64).item()
    b.sirllm_step_ragged_out_of_place(z, tok, w.vocab, scores, held_dev, cu, total, max_cand, pol, k, v, kd, vd, kept, out,
                                      n_keep_dev, max_new=int(n_new.max()))
    torch.cuda.synchronize()
    gs, gkeep = to_np(scores), to_np(n_keep_dev)
    e = ref.score(to_np(z), to_np(tok), vocab=w.vocab)
    assert k.view(torch.int16).sum(dtype=torch.int64).item() == k_sum and v.view(torch.int16).sum(dtype=torch.int64).item() == v_sum
    r0 = 0
    for s in range(S):
        h, n = int(n_held[s]), int(n_new[s])
        assert_scores_close(gs[s, h:h + n], e[r0:r0 + n])
        np.testing.assert_array_equal(gs[s, :h], hs[s, :h])
        r0 += n
        ki, so = ref.decay_select(gs[s:s + 1, :h + n], h, n, ref.Policy(*pol))
        nk = ki.shape[1]
        assert gkeep[s] == nk == min(h + n, budget)
        np.testing.assert_array_equal(to_np(kept)[s, :nk], ki[0])
        np.testing.assert_array_equal(to_np(out)[s, :nk].view(np.uint32), so[0].view(np.uint32))
        rk, rv = ref.compact_kv(to_np(k[s:s + 1].view(torch.int16)), to_np(v[s:s + 1].view(torch.int16)), ki, n_src=h + n)
        gk, gv = to_np(kd[s:s + 1].view(torch.int16)), to_np(vd[s:s + 1].view(torch.int16))
        assert np.array_equal(gk[:, :, :, :nk], rk) and np.array_equal(gv[:, :, :, :nk], rv), f"stream {s}: K/V differ from the oracle"
        pad = torch.tensor(77, dtype=torch.bfloat16).view(torch.int16).item()
        assert (gk[:, :, :, nk:] == pad).all() and (gv[:, :, :, nk:] == pad).all(), f"stream {s}: written past its kept slots"


@pytest.mark.timeout(600)
def test_long_context_step(b, ref):
    """A 128K-slot budget at the Llama-3-8B shape: 133120 candidates (selection by the multi-workgroup path),
    35 GB of K/V read and written.  Scores and the kept set are checked in full, K/V on sampled planes."""
    w = synth.WORKLOADS["llama3_128k"]
    ref.set_threads(16)
    pol = b.Policy(w.n_sink, w.n_topk, w.n_recent, w.decay)
    S, n_held, n_new, n_cand, n_keep = w.n_streams, w.n_held, w.n_new, w.n_cand, w.n_keep
    logits = synth.make_logits(w, turn=1, device=DEV)
    tok = synth.make_token_ids(w, turn=1, device=DEV)
    scores = torch.full((S, n_cand), -3.0, device=DEV)
    held = synth.make_held_scores(w, device=DEV)
    scores[:, :n_held] = held
    k_src = synth.make_kv(w, device=DEV, which="k")
    v_src = synth.make_kv(w, device=DEV, which="v")
    dst_shape = (S, w.n_layers, w.n_kv_heads, n_keep, w.head_dim)
    k_dst = torch.zeros(dst_shape, dtype=k_src.dtype, device=DEV)
    v_dst = torch.zeros(dst_shape, dtype=k_src.dtype, device=DEV)
    kept = torch.full((S, n_keep), -1, dtype=torch.int32, device=DEV)
    out = torch.full((S, n_keep), -1.0, device=DEV)
    ws = torch.zeros(b.sirllm_workspace_bytes(S, n_cand, S * n_new, w.vocab), dtype=torch.uint8, device=DEV)
    assert ws.numel() > 0
    b.sirllm_step(logits, tok, w.vocab, scores, n_held, n_new, pol, k_src, v_src, k_dst, v_dst, kept, out, workspace=ws)
    torch.cuda.synchronize()
    Eg = to_np(scores)
    want = ref.score(to_np(logits), to_np(tok), vocab=w.vocab).reshape(S, n_new)
    assert_scores_close(Eg[:, n_held:], want)
    ri, ro = ref.decay_select(Eg, n_held, n_new, ref.Policy(*pol))
    np.testing.assert_array_equal(to_np(kept), ri)
    np.testing.assert_array_equal(to_np(out).view(np.uint32), ro.view(np.uint32))
    assert ri.shape[1] == w.budget == 131072
    rng = np.random.default_rng(1)
    for _ in range(10):
        l, h = int(rng.integers(w.n_layers)), int(rng.integers(w.n_kv_heads))
        src_t, dst_t = (k_src, k_dst) if rng.integers(2) else (v_src, v_dst)
        rp, _ = ref.compact_kv(to_np(src_t[:, l:l + 1, h:h + 1]), None, ri)
        assert np.array_equal(to_np(dst_t[:, l:l + 1, h:h + 1]), rp), f"plane (layer {l}, head {h}) differs"


@pytest.mark.timeout(900)
def test_batched_dialogue_200_turns(b, ref):
    """32 streams x 200 turns x 256 tokens; scores persist across turns; checked at turns 1, 50, 200: the new
    scores, the kept list, the compacted scores and every byte of the compacted K and V of all 32 streams."""
    from paper_2405_12528_amd.cache import RetentiveCache
    w = synth.WORKLOADS["batched_dialogue"]
    ref.set_threads(16)
    S, n_new = w.n_streams, w.n_new
    pol = (w.n_sink, w.n_topk, w.n_recent, w.decay)
    cache = RetentiveCache(S, w.n_layers, w.n_kv_heads, w.head_dim, pol, max_new=n_new, device=DEV)
    gk = torch.Generator(device=DEV).manual_seed(12345)
    # pinned staging buffers, one per array that is alive at the same time (a stream's K or V is 0.6 GB)
    per_stream = w.n_layers * w.n_kv_heads * w.n_cand * w.head_dim
    stage = [torch.empty(per_stream, dtype=torch.int16, pin_memory=True) for _ in range(4)]

    def staged(t, which):
        """Host copy of a bfloat16 device view with identical bytes, as uint16 bit patterns."""
        c = t.contiguous().view(torch.int16)
        buf = stage[which][:c.numel()].view(c.shape)
        buf.copy_(c)
        return buf.numpy().view(np.uint16)

    for turn in range(1, w.n_turns + 1):
        logits = synth.make_logits(w, turn=turn, device=DEV)
        tok = synth.make_token_ids(w, turn=turn, device=DEV)
        k_new, v_new = cache.new_kv_slots(n_new)
        k_new.copy_(torch.randn(k_new.shape, generator=gk, device=DEV, dtype=torch.float32).to(k_new.dtype))
        v_new.copy_(torch.randn(v_new.shape, generator=gk, device=DEV, dtype=torch.float32).to(v_new.dtype))
        n_held = cache.n_held
        n_cand = n_held + n_new
        assert n_cand == min(turn * n_new, w.n_cand)
        check = turn in w.checked_turns
        if check:   # the pre-step state stays intact: compaction is out of place
            held = cache.scores[:, :n_held].clone()
            k_pre, v_pre, s_pre = cache.k, cache.v, cache.scores
        evicted = cache.step(logits, tok, w.vocab)
        assert evicted == (n_cand > w.budget)
        assert cache.n_held == min(n_cand, w.budget)
        if not check:
            continue
        torch.cuda.synchronize()
        n_keep = cache.n_held
        Eg = to_np(s_pre[:, :n_cand])
        want = ref.score(to_np(logits), to_np(tok), vocab=w.vocab).reshape(S, n_new)
        assert_scores_close(Eg[:, n_held:], want)
        np.testing.assert_array_equal(Eg[:, :n_held].view(np.uint32), to_np(held).view(np.uint32))
        ri, ro = ref.decay_select(Eg, n_held, n_new, ref.Policy(*pol))
        np.testing.assert_array_equal(to_np(cache.kept_idx[:, :n_keep]), ri)
        np.testing.assert_array_equal(to_np(cache.scores[:, :n_keep]).view(np.uint32), ro.view(np.uint32))
        if not evicted:
            assert cache.k.data_ptr() == k_pre.data_ptr()       # the cache stayed where it was
            continue
        assert cache.k.data_ptr() != k_pre.data_ptr()
        # K and V of every stream, whole: the oracle gathers one stream at a time from the pre-step buffers
        # (compaction is out of place, so they still hold the candidates), 1.2 GB per stream
        for s in range(S):
            rk, rv = ref.compact_kv(staged(k_pre[s:s + 1, :, :, :n_cand], 0), staged(v_pre[s:s + 1, :, :, :n_cand], 1),
                                    ri[s:s + 1])
            assert np.array_equal(staged(cache.k[s:s + 1, :, :, :n_keep], 2), rk), f"K of stream {s} differs at turn {turn}"
            assert np.array_equal(staged(cache.v[s:s + 1, :, :, :n_keep], 3), rv), f"V of stream {s} differs at turn {turn}"
            if s % 8 == 7:
                print(f"turn {turn}: K/V of streams 0..{s} checked", flush=True)
        print(f"turn {turn}: checked", flush=True)


@pytest.mark.timeout(600)
def test_rps_dialogue_many_small_turns(b, ref):
    """The paper's own operating point (Sec. 4.2, the Rock-Paper-Scissors dialogues of Table 3): 2000 rounds of
    ~54 tokens, budget 1024 = 4 + 1020 + 0, the cache never reset; with no recent window the selection depends
    on this turn's scores (three dependent launches).  Checked against the oracle at rounds 1, 19, 20 (the first
    eviction), 100, 300, 1000 and 2000; the budget invariant at every round."""
    from paper_2405_12528_amd.cache import RetentiveCache
    w = synth.WORKLOADS["rps_dialogue"]
    ref.set_threads(16)
    pol = (w.n_sink, w.n_topk, w.n_recent, w.decay)
    cache = RetentiveCache(1, w.n_layers, w.n_kv_heads, w.head_dim, pol, max_new=w.n_new, device=DEV)
    gk = torch.Generator(device=DEV).manual_seed(777)
    last = max(w.checked_turns)
    for turn in range(1, last + 1):
        logits = synth.make_logits(w, turn=turn, device=DEV)
        tok = synth.make_token_ids(w, turn=turn, device=DEV)
        k_new, v_new = cache.new_kv_slots(w.n_new)
        k_new.copy_(torch.randn(k_new.shape, generator=gk, device=DEV, dtype=torch.float32).to(k_new.dtype))
        v_new.copy_(torch.randn(v_new.shape, generator=gk, device=DEV, dtype=torch.float32).to(v_new.dtype))
        n_held = cache.n_held
        n_cand = n_held + w.n_new
        check = turn in w.checked_turns
        if check:
            held = cache.scores[:, :n_held].clone()
            k_pre, v_pre, s_pre = cache.k, cache.v, cache.scores
        evicted = cache.step(logits, tok, w.vocab)
        assert evicted == (turn * w.n_new > w.budget)
        assert cache.n_held == min(turn * w.n_new, w.budget)
        if not check:
            continue
        torch.cuda.synchronize()
        n_keep = cache.n_held
        Eg = to_np(s_pre[:, :n_cand])
        want = ref.score(to_np(logits), to_np(tok), vocab=w.vocab).reshape(1, w.n_new)
        assert_scores_close(Eg[:, n_held:], want)
        np.testing.assert_array_equal(Eg[:, :n_held].view(np.uint32), to_np(held).view(np.uint32))
        ri, ro = ref.decay_select(Eg, n_held, w.n_new, ref.Policy(*pol))
        np.testing.assert_array_equal(to_np(cache.kept_idx[:, :n_keep]), ri)
        np.testing.assert_array_equal(to_np(cache.scores[:, :n_keep]).view(np.uint32), ro.view(np.uint32))
        if evicted:
            rk, rv = ref.compact_kv(to_np(k_pre[:, :, :, :n_cand]), to_np(v_pre[:, :, :, :n_cand]), ri)
            assert np.array_equal(to_np(cache.k[:, :, :, :n_keep]), rk)
            assert np.array_equal(to_np(cache.v[:, :, :, :n_keep]), rv)
            assert n_keep == w.budget and ri[0, :4].tolist() == [0, 1, 2, 3]
        print(f"turn {turn}: checked (evicted={evicted})", flush=True)


def test_dailydialog_shaped_dialogues_with_resets(b, ref):
    """The paper's everyday-dialogue setting (Sec. 4.2, Table 1): budget 512 = 4 + 508 + 0, decay 0.6, the cache reset
    after every dialogue.  Synthetic stand-in for the dataset: 24 dialogues of 3 to 5 turns whose token totals are
    spread around the paper's mean of ~460 so that about a third of them outgrow the 512 slots (those are the
    dialogues the method is for); turns of unequal length.  Every turn of every dialogue is checked in full."""
    from paper_2405_12528_amd.cache import RetentiveCache
    V, L, H, D = 32000, 2, 2, 64
    pol = (4, 508, 0, 0.6)
    rng = np.random.default_rng(461)
    g0 = torch.Generator(device=DEV).manual_seed(55)
    cache = RetentiveCache(1, L, H, D, pol, max_new=400, device=DEV)
    outgrew = 0
    for dialogue in range(24):
        cache.reset()
        turns = int(rng.integers(3, 6))
        total = int(np.clip(rng.lognormal(np.log(430.0), 0.45), 120, 1500))
        cuts = np.sort(rng.choice(np.arange(1, total), size=turns - 1, replace=False))
        lens = np.diff(np.concatenate([[0], cuts, [total]]))
        lens = np.minimum(lens, 400)
        outgrew += int(lens.sum() > 512)
        for n_new in (int(x) for x in lens):
            z = (torch.randn((n_new, V), generator=g0, device=DEV) * 3.0).to(torch.bfloat16)
            tok = torch.randint(0, V, (n_new,), generator=g0, device=DEV, dtype=torch.int32)
            k_new, v_new = cache.new_kv_slots(n_new)
            k_new.copy_(torch.randn(k_new.shape, generator=g0, device=DEV).to(k_new.dtype))
            v_new.copy_(torch.randn(v_new.shape, generator=g0, device=DEV).to(v_new.dtype))
            n_held = cache.n_held
            n_cand = n_held + n_new
            held = cache.scores[:, :n_held].clone()
            k_pre, v_pre, s_pre = cache.k, cache.v, cache.scores
            evicted = cache.step(z, tok, V)
            torch.cuda.synchronize()
            assert evicted == (n_cand > 512) and cache.n_held == min(n_cand, 512)
            n_keep = cache.n_held
            Eg = to_np(s_pre[:, :n_cand])
            assert_scores_close(Eg[0, n_held:], ref.score(to_np(z), to_np(tok), vocab=V))
            np.testing.assert_array_equal(Eg[:, :n_held].view(np.uint32), to_np(held).view(np.uint32))
            ri, ro = ref.decay_select(Eg, n_held, n_new, ref.Policy(*pol))
            np.testing.assert_array_equal(to_np(cache.kept_idx[:, :n_keep]), ri)
            np.testing.assert_array_equal(to_np(cache.scores[:, :n_keep]).view(np.uint32), ro.view(np.uint32))
            if evicted:
                rk, rv = ref.compact_kv(to_np(k_pre[:, :, :, :n_cand]), to_np(v_pre[:, :, :, :n_cand]), ri)
                assert np.array_equal(to_np(cache.k[:, :, :, :n_keep]), rk)
                assert np.array_equal(to_np(cache.v[:, :, :, :n_keep]), rv)
            else:
                assert torch.equal(cache.k[:, :, :, :n_cand], k_pre[:, :, :, :n_cand])
    assert 4 <= outgrew <= 16, outgrew


def test_per_layer_cache_dialogues(b, ref):
    """LayeredRetentiveCache: K and V as one tensor per layer, stepped by sirllm_score_select and compacted in place
    by sirllm_compact_kv_inplace_layers.  Eight synthetic dialogues with resets in between (budget 512 = 4 + 380 +
    128: some turns fit the recent window and share a launch for scoring and selection, some do not); every turn is
    checked against the oracle fed the GPU's scores, layer by layer."""
    from paper_2405_12528_amd.cache import LayeredRetentiveCache
    V, L, H, D, S = 5000, 3, 2, 64, 2
    pol = (4, 380, 128, 0.7)
    rng = np.random.default_rng(99)
    g0 = torch.Generator(device=DEV).manual_seed(17)
    cache = LayeredRetentiveCache(S, L, H, D, pol, max_new=300, device=DEV)
    evictions = 0
    for dialogue in range(8):
        cache.reset()
        for n_new in (int(x) for x in rng.integers(20, 300, size=int(rng.integers(3, 7)))):
            z = (torch.randn((S * n_new, V), generator=g0, device=DEV) * 3.0).to(torch.bfloat16)
            tok = torch.randint(0, V, (S * n_new,), generator=g0, device=DEV, dtype=torch.int32)
            for l in range(L):
                k_new, v_new = cache.new_kv_slots(l, n_new)
                k_new.copy_(torch.randn(k_new.shape, generator=g0, device=DEV).to(k_new.dtype))
                v_new.copy_(torch.randn(v_new.shape, generator=g0, device=DEV).to(v_new.dtype))
            n_held = cache.n_held
            n_cand = n_held + n_new
            held = cache.scores[:, :n_held].clone()
            k_pre = [to_np(t[:, :, :n_cand])[:, None].copy() for t in cache.k]
            v_pre = [to_np(t[:, :, :n_cand])[:, None].copy() for t in cache.v]
            s_pre = cache.scores
            evicted = cache.step(z, tok, V)
            torch.cuda.synchronize()
            evictions += int(evicted)
            assert evicted == (n_cand > 512) and cache.n_held == min(n_cand, 512)
            n_keep = cache.n_held
            Eg = to_np(s_pre[:, :n_cand])
            assert_scores_close(Eg[:, n_held:].reshape(-1), ref.score(to_np(z), to_np(tok), vocab=V))
            np.testing.assert_array_equal(Eg[:, :n_held].view(np.uint32), to_np(held).view(np.uint32))
            ri, ro = ref.decay_select(Eg, n_held, n_new, ref.Policy(*pol))
            np.testing.assert_array_equal(to_np(cache.kept_idx[:, :n_keep]), ri)
            np.testing.assert_array_equal(to_np(cache.scores[:, :n_keep]).view(np.uint32), ro.view(np.uint32))
            for l in range(L):
                if evicted:
                    ref.compact_kv_inplace(k_pre[l], v_pre[l], ri, n_src=n_cand)
                assert np.array_equal(to_np(cache.k[l][:, :, :n_cand]), k_pre[l][:, 0]), f"layer {l}: K differs"
                assert np.array_equal(to_np(cache.v[l][:, :, :n_cand]), v_pre[l][:, 0]), f"layer {l}: V differs"
    assert evictions >= 5


def test_step_replays_from_a_captured_graph(b, ref):
    """sirllm_step allocates nothing, synchronises nothing and clears nothing with memset nodes, so it
    can be captured into a HIP graph; every replay must reproduce the eager result, also with eager
    work and synchronisations between replays."""
    w = synth.WORKLOADS["tiny"]
    pol = b.Policy(4, 30, 0, 0.8)                       # no recent window: the three-launch path
    S, n_held, n_new, V = 2, 60, 40, 777
    g0 = torch.Generator(device=DEV).manual_seed(5)
    z = torch.randn((S * n_new, V), generator=g0, device=DEV) * 2
    tok = torch.randint(0, V, (S * n_new,), generator=g0, device=DEV, dtype=torch.int32)
    held = torch.rand((S, n_held), generator=g0, device=DEV) * 6
    k_c = torch.randn((S, 2, 2, n_held + n_new, 16), generator=g0, device=DEV)
    v_c = torch.randn((S, 2, 2, n_held + n_new, 16), generator=g0, device=DEV)
    n_keep = 34

    def fresh():
        E = torch.zeros((S, n_held + n_new), device=DEV)
        E[:, :n_held] = held
        return dict(E=E, idx=torch.zeros((S, n_keep), dtype=torch.int32, device=DEV),
                    out=torch.zeros((S, n_keep), device=DEV), k=torch.zeros((S, 2, 2, n_keep, 16), device=DEV),
                    v=torch.zeros((S, 2, 2, n_keep, 16), device=DEV))

    def run(t):
        b.sirllm_step(z, tok, V, t["E"], n_held, n_new, pol, k_c, v_c, t["k"], t["v"], t["idx"], t["out"])

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
        for t in cap.values():                           # eager work between replays: wipe every output
            t.zero_() if t is not cap["E"] else t[:, n_held:].zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name in eager:
            assert torch.equal(cap[name], eager[name]), f"replay {rep}: {name} differs from the eager run"


def test_per_layer_step_replays_from_a_captured_graph(b):
    """sirllm_score_select + sirllm_compact_kv_layers (the per-layer pointer table travels in the kernel arguments, so
    nothing is staged or allocated) captured into a HIP graph: every replay reproduces the eager result."""
    pol = b.Policy(4, 22, 8, 0.8)
    S, L, H, D, n_held, n_new, V, n_keep = 2, 3, 2, 16, 60, 40, 777, 34
    g0 = torch.Generator(device=DEV).manual_seed(6)
    z = torch.randn((S * n_new, V), generator=g0, device=DEV) * 2
    tok = torch.randint(0, V, (S * n_new,), generator=g0, device=DEV, dtype=torch.int32)
    held = torch.rand((S, n_held), generator=g0, device=DEV) * 6
    k_c = [torch.randn((S, H, n_held + n_new, D), generator=g0, device=DEV) for _ in range(L)]
    v_c = [torch.randn((S, H, n_held + n_new, D), generator=g0, device=DEV) for _ in range(L)]

    def fresh():
        E = torch.zeros((S, n_held + n_new), device=DEV)
        E[:, :n_held] = held
        t = dict(E=E, idx=torch.zeros((S, n_keep), dtype=torch.int32, device=DEV), out=torch.zeros((S, n_keep), device=DEV))
        for l in range(L):
            t[f"k{l}"] = torch.zeros((S, H, n_keep, D), device=DEV)
            t[f"v{l}"] = torch.zeros((S, H, n_keep, D), device=DEV)
        return t

    def run(t):
        assert b.sirllm_score_select(z, tok, V, t["E"], n_held, n_new, pol, t["idx"], t["out"]) == n_keep
        b.sirllm_compact_kv_layers(k_c, v_c, [t[f"k{l}"] for l in range(L)], [t[f"v{l}"] for l in range(L)], t["idx"], n_keep,
                                   n_src=n_held + n_new)

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
    for rep in range(3):
        for name, t in cap.items():                      # eager work between replays: wipe every output
            t.zero_() if name != "E" else t[:, n_held:].zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name in eager:
            assert torch.equal(cap[name], eager[name]), f"replay {rep}: {name} differs from the eager run"
    assert eager["k0"].abs().sum() > 0


@pytest.mark.parametrize("kind", ["logits", "hidden states", "two buffers", "two buffers, hidden states"])
def test_ragged_dialogues_of_unequal_length(b, ref, kind):
    """Six dialogues in one serving batch, each with its own arrival turn and its own number of tokens per
    turn (some turns idle), stepped together by sirllm_step_ragged (or, fed with hidden states and the output
    embedding matrix, by sirllm_step_lmhead_ragged) with in-place compaction, or by sirllm_step_ragged_out_of_place (fed with
    hidden states: sirllm_step_lmhead_ragged_out_of_place) between two buffer pairs that swap every step; the oracle replays every stream on its own and every turn is
    compared in full."""
    from paper_2405_12528_amd.cache import RaggedRetentiveCache, RaggedTwoBufferCache
    from_hidden = kind.endswith("hidden states")
    S, L, H, D, V = 6, 2, 2, 16, 400
    pol = (4, 20, 8, 0.9)
    rng = np.random.default_rng(11)
    make = RaggedTwoBufferCache if kind.startswith("two buffers") else RaggedRetentiveCache
    cache = make(S, L, H, D, pol, max_new=40, kv_dtype=torch.float32, device=DEV)
    g0 = torch.Generator(device=DEV).manual_seed(3)
    d_model = 64
    emb = (torch.randn((V, d_model), generator=g0, device=DEV) * (2.5 / d_model ** 0.5)).to(torch.bfloat16)
    # oracle state per stream
    oE = [np.zeros((1, 0), np.float32) for _ in range(S)]
    oK = [np.zeros((1, L, H, 0, D), np.float32) for _ in range(S)]
    oV = [np.zeros((1, L, H, 0, D), np.float32) for _ in range(S)]
    arrival = [1, 1, 3, 5, 8, 12]
    for turn in range(1, 31):
        n_new = [0 if turn < arrival[s] or rng.random() < 0.2 else int(rng.integers(1, 41)) for s in range(S)]
        if turn == 20:
            cache.reset(2)                                        # stream 2 starts a new dialogue
            oE[2], oK[2], oV[2] = oE[2][:, :0], oK[2][:, :, :, :0], oV[2][:, :, :, :0]
        total = sum(n_new)
        z = torch.randn((total, V), generator=g0, device=DEV) * 2.5
        hid = (torch.randn((total, d_model), generator=g0, device=DEV) + 0.5).to(torch.bfloat16)
        tok = torch.randint(0, V, (total,), generator=g0, device=DEV, dtype=torch.int32)
        new_kv = []
        for s in range(S):
            ks, vs = cache.new_kv_slots(s, n_new[s])
            ks.copy_(torch.randn(ks.shape, generator=g0, device=DEV))
            vs.copy_(torch.randn(vs.shape, generator=g0, device=DEV))
            new_kv.append((to_np(ks)[None], to_np(vs)[None]))
        held_before = list(cache.n_held)
        pre_scores = cache.scores                                   # new scores are appended to this array
        evicted = cache.step_from_hidden(hid, emb, tok, n_new) if from_hidden else cache.step(z, tok, V, n_new)
        torch.cuda.synchronize()
        zs, ts = to_np(z), to_np(tok)
        r0 = 0
        for s in range(S):
            h, n = held_before[s], n_new[s]
            assert h == oE[s].shape[1]
            Kc = np.concatenate([oK[s], new_kv[s][0]], axis=3)
            Vc = np.concatenate([oV[s], new_kv[s][1]], axis=3)
            if h + n == 0:
                continue
            # scores within tolerance, then the oracle's selection and gather on the GPU's scores
            g_new = to_np(pre_scores[s, h:h + n])
            if n and from_hidden:
                assert_scores_close(g_new, ref.lmhead_score(np.ascontiguousarray(to_np(hid)[r0:r0 + n]), to_np(emb),
                                                            ts[r0:r0 + n]), atol=2e-5)
            elif n:
                assert_scores_close(g_new, ref.score(np.ascontiguousarray(zs[r0:r0 + n]), ts[r0:r0 + n], vocab=V))
            r0 += n
            cand = np.concatenate([oE[s], g_new[None]], axis=1)
            ki, so = ref.decay_select(cand, h, n, ref.Policy(*pol))
            n_keep = ki.shape[1]
            assert cache.n_held[s] == n_keep and evicted[s] == (h + n > 32)
            np.testing.assert_array_equal(to_np(cache.kept_idx[s, :n_keep]), ki[0])
            np.testing.assert_array_equal(to_np(cache.scores[s, :n_keep]).view(np.uint32), so[0].view(np.uint32))
            rk, rv = ref.compact_kv(Kc, Vc, ki)
            assert np.array_equal(to_np(cache.k[s:s + 1, :, :, :n_keep]), rk), f"turn {turn} stream {s}: K differs"
            assert np.array_equal(to_np(cache.v[s:s + 1, :, :, :n_keep]), rv), f"turn {turn} stream {s}: V differs"
            oE[s], oK[s], oV[s] = so, rk, rv


def test_ragged_cache_beyond_one_workgroups_slots(b, ref):
    """RaggedRetentiveCache with a budget of 33000 slots: once a stream may hold more than 32768 slots the batch is
    selected by the multi-workgroup kernels (workspace from the cache).  Two streams fill at different speeds, so
    early steps keep everything, later ones evict in one stream only, then in both; the oracle replays every step."""
    from paper_2405_12528_amd.cache import RaggedRetentiveCache
    S, L, H, D, V = 2, 1, 2, 8, 200
    pol = (4, 32000, 996, 0.9)
    rng = np.random.default_rng(33)
    cache = RaggedRetentiveCache(S, L, H, D, pol, max_new=3000, kv_dtype=torch.float32, device=DEV)
    g0 = torch.Generator(device=DEV).manual_seed(9)
    oE = [np.zeros((1, 0), np.float32) for _ in range(S)]
    oK = [np.zeros((1, L, H, 0, D), np.float32) for _ in range(S)]
    oV = [np.zeros((1, L, H, 0, D), np.float32) for _ in range(S)]
    seen_evictions = [0, 0]
    for turn in range(1, 21):
        n_new = [3000, int(rng.integers(1500, 2600))]
        total = sum(n_new)
        z = torch.randn((total, V), generator=g0, device=DEV) * 2.5
        tok = torch.randint(0, V, (total,), generator=g0, device=DEV, dtype=torch.int32)
        new_kv = []
        for s in range(S):
            ks, vs = cache.new_kv_slots(s, n_new[s])
            ks.copy_(torch.randn(ks.shape, generator=g0, device=DEV))
            vs.copy_(torch.randn(vs.shape, generator=g0, device=DEV))
            new_kv.append((to_np(ks)[None], to_np(vs)[None]))
        held_before = list(cache.n_held)
        pre_scores = cache.scores
        evicted = cache.step(z, tok, V, n_new)
        torch.cuda.synchronize()
        zs, ts = to_np(z), to_np(tok)
        r0 = 0
        for s in range(S):
            h, n = held_before[s], n_new[s]
            Kc = np.concatenate([oK[s], new_kv[s][0]], axis=3)
            Vc = np.concatenate([oV[s], new_kv[s][1]], axis=3)
            g_new = to_np(pre_scores[s, h:h + n])
            assert_scores_close(g_new, ref.score(np.ascontiguousarray(zs[r0:r0 + n]), ts[r0:r0 + n], vocab=V))
            r0 += n
            ki, so = ref.decay_select(np.concatenate([oE[s], g_new[None]], axis=1), h, n, ref.Policy(*pol))
            n_keep = ki.shape[1]
            assert cache.n_held[s] == n_keep and evicted[s] == (h + n > 33000)
            seen_evictions[s] += int(evicted[s])
            np.testing.assert_array_equal(to_np(cache.kept_idx[s, :n_keep]), ki[0])
            np.testing.assert_array_equal(to_np(cache.scores[s, :n_keep]).view(np.uint32), so[0].view(np.uint32))
            rk, rv = ref.compact_kv(Kc, Vc, ki)
            assert np.array_equal(to_np(cache.k[s:s + 1, :, :, :n_keep]), rk), f"turn {turn} stream {s}: K differs"
            assert np.array_equal(to_np(cache.v[s:s + 1, :, :, :n_keep]), rv), f"turn {turn} stream {s}: V differs"
            oE[s], oK[s], oV[s] = so, rk, rv
    assert seen_evictions[0] >= 8 and 1 <= seen_evictions[1] < seen_evictions[0]


def test_c_example_runs_without_torch():
    """examples/step_example.c: the C ABI driven from plain C with the HIP runtime only."""
    import os
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = os.path.join(root, "examples", "step_example")
    if not os.path.exists(exe):                     # built by build(); compile it here only if nothing is there
        from paper_2405_12528_amd import build
        build.build_example()
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stderr
    assert r.stdout.startswith("ok: libsirllm")


@pytest.mark.timeout(300)
def test_score_rows_beyond_4_gib(b, ref):
    """Row offsets need 64 bits: 9000 rows x 128256 fp32 logits are 4.6 GB; the oracle checks the first
    rows, rows on either side of the 2 GiB and 4 GiB marks, and the last rows."""
    V, n_rows = 128256, 9000
    g0 = torch.Generator(device=DEV).manual_seed(1)
    z = torch.empty((n_rows, V), device=DEV)
    for r0 in range(0, n_rows, 1000):
        z[r0:r0 + 1000] = torch.randn((min(1000, n_rows - r0), V), generator=g0, device=DEV) * 3
    tok = torch.randint(0, V, (n_rows,), generator=g0, device=DEV, dtype=torch.int32)
    out = torch.zeros(n_rows, device=DEV)
    b.sirllm_score(z, tok, out)
    torch.cuda.synchronize()
    per_row = V * 4
    marks = sorted({0, 1, (2 << 30) // per_row, (2 << 30) // per_row + 1, (4 << 30) // per_row, (4 << 30) // per_row + 1,
                    n_rows - 2, n_rows - 1})
    rows = torch.tensor(marks, device=DEV)
    want = ref.score(to_np(z[rows]), to_np(tok[rows]))
    assert_scores_close(to_np(out[rows]), want)


def test_python_example_runs_both_routes():
    """examples/dialogue_loop.py: six turns through RetentiveCache from logits and from the LM head; the sinks stay
    the first four tokens of the dialogue and the cache holds the budget."""
    import importlib.util
    path = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "examples", "dialogue_loop.py")
    spec = importlib.util.spec_from_file_location("dialogue_loop", path)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    for extra in ([], ["--from-hidden"]):
        origin = mod.main(["--turns", "6"] + extra)
        assert origin.shape == (32, 2)
        assert origin[-8:, 0].tolist() == [6] * 8           # the recent window is the end of the last turn


def _independent_job(seed, S, n_held, n_new, V, pol_t, D):
    """Inputs and zeroed outputs of one step, all its own."""
    g = torch.Generator(device=DEV).manual_seed(seed)
    n_cand = n_held + n_new
    n_keep = min(n_cand, pol_t[0] + pol_t[1] + pol_t[2])
    E = torch.zeros((S, n_cand), device=DEV)
    E[:, :n_held] = torch.rand((S, n_held), generator=g, device=DEV) * 6
    return dict(z=torch.randn((S * n_new, V), generator=g, device=DEV) * 2,
                tok=torch.randint(0, V, (S * n_new,), generator=g, device=DEV, dtype=torch.int32),
                E=E, k=torch.randn((S, 2, 3, n_cand, D), generator=g, device=DEV),
                v=torch.randn((S, 2, 3, n_cand, D), generator=g, device=DEV),
                kd=torch.zeros((S, 2, 3, n_keep, D), device=DEV), vd=torch.zeros((S, 2, 3, n_keep, D), device=DEV),
                idx=torch.zeros((S, n_keep), dtype=torch.int32, device=DEV), out=torch.zeros((S, n_keep), device=DEV),
                shape=(V, n_held, n_new), pol=pol_t)


def _run_job(b, j, stream=None):
    V, n_held, n_new = j["shape"]
    b.sirllm_step(j["z"], j["tok"], V, j["E"], n_held, n_new, b.Policy(*j["pol"]), j["k"], j["v"], j["kd"], j["vd"],
                  j["idx"], j["out"], stream=stream)


_JOBS = [(11, 2, 3000, 500, 5003, (4, 1500, 500, 0.9), 64), (12, 1, 700, 300, 32000, (4, 400, 100, 0.8), 128),
         (13, 3, 100, 40, 777, (4, 50, 8, 0.9), 16), (14, 1, 6000, 2000, 1000, (4, 2044, 2048, 0.9), 32)]


def test_steps_on_two_streams_at_once_do_not_disturb_each_other(b):
    """The library keeps no state between calls: independent steps enqueued on two streams, interleaved, give
    the bytes the same steps give one after the other."""
    want = [_independent_job(*a) for a in _JOBS]
    for j in want:
        _run_job(b, j)
    torch.cuda.synchronize()
    got = [_independent_job(*a) for a in _JOBS]
    torch.cuda.synchronize()
    s0, s1 = torch.cuda.Stream(), torch.cuda.Stream()
    for rep in range(3):
        for i, j in enumerate(got):
            _run_job(b, j, stream=(s0, s1)[i % 2])
    torch.cuda.synchronize()
    for w, g in zip(want, got):
        for name in ("E", "kd", "vd", "idx", "out"):
            assert torch.equal(w[name], g[name]), f"{name} differs when two streams run at once"


def test_steps_from_two_host_threads_at_once(b):
    """Two host threads calling into the library at the same time, each on a stream of its own."""
    import threading
    want = [_independent_job(*a) for a in _JOBS]
    for j in want:
        _run_job(b, j)
    torch.cuda.synchronize()
    got = [_independent_job(*a) for a in _JOBS]
    torch.cuda.synchronize()
    errors = []

    def worker(jobs):
        try:
            torch.cuda.set_device(0)
            s = torch.cuda.Stream()
            for _ in range(20):
                for j in jobs:
                    _run_job(b, j, stream=s)
            s.synchronize()
        except Exception as e:                                   # surfaced in the main thread below
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(got[0::2],)), threading.Thread(target=worker, args=(got[1::2],))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    torch.cuda.synchronize()
    for w, g in zip(want, got):
        for name in ("E", "kd", "vd", "idx", "out"):
            assert torch.equal(w[name], g[name]), f"{name} differs when two host threads call at once"
