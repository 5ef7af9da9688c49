"""Parity of the HIP path with the CPU oracle, through the C ABI, on one MI355X.

Scores: |gpu - ref| <= 1e-6 + 1e-5*|ref| (binary32 accumulation against the oracle's double).
Kept indices, compacted scores and compacted K/V: bit exact, with the oracle fed the GPU's own
scores where a selection depends on them (both sides then decide on identical binary32 values).
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


def assert_scores_close(gpu: np.ndarray, want: np.ndarray, atol: float = 1e-6):
    """atol: 1e-6 for scores from stored logits; 2e-5 for scores from the LM head, whose logits are binary32 sums of
    d_model products (derivation at the top of test_gpu_lmhead.py)."""
    nan_w, nan_g = np.isnan(want), np.isnan(gpu)
    np.testing.assert_array_equal(nan_g, nan_w)
    inf_w = np.isinf(want)
    np.testing.assert_array_equal(gpu[inf_w], want[inf_w])
    ok = ~(nan_w | inf_w)
    err = np.abs(gpu[ok].astype(np.float64) - want[ok].astype(np.float64))
    tol = atol + 1e-5 * np.abs(want[ok].astype(np.float64))
    bad = err > tol
    assert not bad.any(), f"{bad.sum()} scores off; worst {err.max():.3e} (tolerance {tol[err.argmax()]:.3e})"


def gpu_score(b, z: torch.Tensor, tok: torch.Tensor, vocab=None):
    out = torch.full((z.shape[0],), -12345.0, dtype=torch.float32, device=DEV)
    b.sirllm_score(z, tok, out, vocab=vocab)
    torch.cuda.synchronize()
    return to_np(out)


# ------------------------------------------------------------------------------------- score
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16])
@pytest.mark.parametrize("n_rows,V,ld", [
    (64, 1000, 1000),        # the tiny workload's shape
    (37, 2311, 2311),        # odd length: rows start at every alignment, scalar head and tail
    (9, 4099, 4200),         # padded rows
    (3, 1, 1), (4, 3, 3), (5, 7, 9), (6, 17, 17), (2, 255, 255), (2, 4096, 4096), (2, 4097, 4097),
    (5, 32000, 32000),       # several sweeps of a 1024-thread workgroup and a ragged last sweep
    (3, 128256, 128256),
    (1100, 515, 520),        # 512-thread workgroups
    (2100, 300, 300),        # 256-thread workgroups
])
def test_score_matches_oracle(b, ref, dtype, n_rows, V, ld):
    g = torch.Generator(device=DEV).manual_seed(n_rows * 7919 + V)
    z = torch.randn((n_rows, ld), generator=g, device=DEV) * 3.0
    z[::3, V // 2] += 8.0
    if ld > V:
        z[:, V:] = 1.0e4
    if ld > V and dtype == torch.float16:
        z[:, V:] = 6.0e4                                   # the padding sentinel must fit binary16
    z = z.to(dtype)
    tok = torch.randint(0, V, (n_rows,), generator=g, device=DEV, dtype=torch.int32)
    got = gpu_score(b, z, tok, vocab=V)
    want = ref.score(to_np(z), to_np(tok), vocab=V)
    assert_scores_close(got, want)


def test_score_workload_generators(b, ref):
    for name, rows in (("tiny", 64), ("llama2_7b", 48), ("llama3_8b", 24)):
        w = synth.WORKLOADS[name]
        z = synth.make_logits(w, turn=1, device=DEV, n_rows=rows)
        tok = synth.make_token_ids(w, turn=1, device=DEV, n_rows=rows)
        assert_scores_close(gpu_score(b, z, tok), ref.score(to_np(z), to_np(tok)))


def test_score_closed_forms(b):
    for V in (1000, 32000, 128256):
        z = torch.full((2, V), -3.25, device=DEV)
        tok = torch.tensor([0, V - 1], dtype=torch.int32, device=DEV)
        np.testing.assert_allclose(gpu_score(b, z, tok), np.log(V), rtol=1e-6)
        np.testing.assert_allclose(gpu_score(b, z.to(torch.bfloat16), tok), np.log(V), rtol=1e-6)
    z = torch.zeros((1, 1000), device=DEV)
    z[0, 123] = 60.0
    assert gpu_score(b, z, torch.tensor([123], dtype=torch.int32, device=DEV))[0] == 0.0


def test_score_non_finite_and_bad_tokens(b, ref):
    V = 600
    z = torch.zeros((8, V), device=DEV)
    z[0, 3] = -np.inf
    z[1, 3] = -np.inf
    z[2, :] = -np.inf
    z[3, 5] = np.inf
    z[4, 7] = np.nan
    z[5, :300] = -np.inf          # whole lanes see nothing finite, others do
    z[6, 300:] = -np.inf
    tok = torch.tensor([0, 3, 0, 0, 0, 400, 10, V], dtype=torch.int32, device=DEV)
    got = gpu_score(b, z, tok)
    want = ref.score(to_np(z), to_np(tok))
    assert_scores_close(got, want)
    assert got[1] == np.inf and np.isnan(got[[2, 3, 4, 7]]).all()
    for dt in (torch.bfloat16, torch.float16):
        zb = z.to(dt)
        assert_scores_close(gpu_score(b, zb, tok), ref.score(to_np(zb), to_np(tok)))


def test_score_binary16_subnormals_and_extremes(b, ref):
    # all finite binary16 values in one row, including subnormals and +-65504
    bits = torch.arange(0, 1 << 16, dtype=torch.int32)
    h = bits.to(torch.int16).view(torch.float16)
    h = h[torch.isfinite(h)]
    z = h[None, :].repeat(3, 1).contiguous().to(DEV)
    z[1] = z[1] / 8                                        # a row whose maximum is not the format's maximum
    z[2, : z.shape[1] // 2] = 0
    tok = torch.tensor([5, 40000, 1], dtype=torch.int32, device=DEV)
    assert_scores_close(gpu_score(b, z, tok), ref.score(to_np(z), to_np(tok)))


def test_score_empty(b):
    z = torch.zeros((0, 16), device=DEV)
    b.sirllm_score(z, torch.zeros(0, dtype=torch.int32, device=DEV), torch.zeros(0, device=DEV))
    torch.cuda.synchronize()


# ------------------------------------------------------------------------------ decay + select
def gpu_select(b, E: np.ndarray, n_held, n_new, pol, pad=3):
    n_streams, n_cand = E.shape
    n_keep = min(n_cand, pol.n_sink + pol.n_topk + pol.n_recent)
    Ed = torch.full((n_streams, n_cand + pad), 777.0, device=DEV)
    Ed[:, :n_cand] = torch.from_numpy(E).to(DEV)
    idx = torch.full((n_streams, n_keep + pad), -7, dtype=torch.int32, device=DEV)
    out = torch.full((n_streams, n_keep + pad), -7.0, device=DEV)
    b.sirllm_decay_select(Ed, n_held, n_new, pol, idx, out)
    torch.cuda.synchronize()
    idx, out = to_np(idx), to_np(out)
    assert (idx[:, n_keep:] == -7).all() and (out[:, n_keep:] == -7.0).all()      # nothing written past n_keep
    return idx[:, :n_keep], out[:, :n_keep]


def check_select(b, ref, E, n_held, n_new, pol):
    gi, go = gpu_select(b, E, n_held, n_new, pol)
    ri, ro = ref.decay_select(E, n_held, n_new, ref.Policy(*pol))
    np.testing.assert_array_equal(gi, ri)
    np.testing.assert_array_equal(go.view(np.uint32), ro.view(np.uint32))


SELECT_CASES = [
    # n_streams, n_held, n_new, n_sink, k, n_recent, decay, levels (0 = continuous)
    (1, 32, 64, 4, 20, 8, 0.9, 0),            # tiny workload, steady state
    (1, 0, 64, 4, 20, 8, 0.9, 0),             # tiny workload, first turn
    (3, 100, 50, 4, 30, 10, 0.9, 5),          # heavy ties
    (2, 3584, 512, 4, 1532, 512, 0.9, 0),     # llama-2 shape
    (2, 7168, 1024, 4, 3068, 1024, 0.85, 40), # mistral shape, ties
    (1, 6144, 2048, 4, 2044, 2048, 0.9, 0),   # llama-3 shape
    (4, 2048, 256, 4, 1788, 256, 0.9, 0),     # batched dialogue shape
    (2, 1000, 24, 4, 1020, 0, 1.0, 0),        # the paper's own setting: 1024 = 4 + 1020 + 0, eta = 1
    (2, 500, 54, 4, 508, 0, 0.7, 0),          # 512 = 4 + 508 + 0
    (1, 40, 10, 0, 7, 0, 0.5, 3),             # no sink, no recent
    (1, 40, 10, 4, 0, 6, 0.5, 0),             # k = 0: StreamLLM
    (1, 40, 10, 0, 0, 6, 0.5, 0),             # sliding window
    (1, 40, 10, 4, 1, 0, 0.5, 2),
    (1, 30, 10, 4, 35, 1, 0.9, 0),            # k = all but one middle slot
    (2, 20, 12, 4, 20, 8, 0.9, 0),            # n_cand == budget
    (2, 10, 5, 4, 20, 8, 0.9, 0),             # n_cand < budget
    (1, 1, 0, 1, 0, 0, 0.9, 0),
    (1, 1020, 5, 4, 100, 8, 0.9, 0),          # crosses the 1024-slot boundary (two slots per thread)
    (1, 32700, 68, 4, 16000, 68, 0.9, 1000),  # the largest size, ragged
    (2, 20000, 0, 4, 9000, 100, 0.99, 0),     # no new tokens at all
    # 8193..16384 slots: sixteen slots per thread (select_kernel<1024, 16>)
    (1, 8000, 193, 4, 4000, 193, 0.9, 0),     # 8193 slots, the first size of that instance
    (2, 11000, 1000, 4, 6000, 500, 0.9, 0),   # 12000 slots, new tokens compete (n_new > n_recent)
    (2, 11500, 800, 4, 5000, 1024, 0.85, 12), # 12300 slots, a dozen score levels: ties across the k-th boundary
    (1, 16000, 384, 4, 16000, 0, 1.0, 3),     # 16384 slots, the last size; no recent window, eta = 1
    (3, 12000, 0, 0, 1, 0, 0.5, 2),           # k = 1 of two levels: the lowest slot of the upper level
    # 16385..32768 slots: thirty-two slots per thread (select_kernel<1024, 32>)
    (1, 16001, 384, 4, 8000, 384, 0.9, 0),    # 16385 slots, the first size of that instance
    (2, 24000, 2000, 4, 13000, 1000, 0.9, 25),
]


@pytest.mark.parametrize("case", SELECT_CASES, ids=[str(c[:6]) for c in SELECT_CASES])
def test_decay_select_matches_oracle(b, ref, case):
    """One workgroup per stream keeps ceil(n_cand / 1024) slots per thread, rounded up to 1, 2, 4, 8, 16 or 32: the
    cases cover every one of those instances of the kernel, each at a first / last size and with ties."""
    n_streams, n_held, n_new, n_sink, k, n_recent, decay, levels = case
    rng = np.random.default_rng(n_held * 31 + n_new)
    n_cand = n_held + n_new
    if levels:
        E = (rng.integers(0, levels, (n_streams, n_cand)) / 8.0).astype(np.float32)
    else:
        E = rng.gamma(2.0, 2.0, (n_streams, n_cand)).astype(np.float32)
    check_select(b, ref, E, n_held, n_new, b.Policy(n_sink, k, n_recent, decay))


def test_decay_select_adversarial_values(b, ref):
    pol = b.Policy(2, 5, 2, 0.5)
    n = 64
    # all equal: pure tie-break
    check_select(b, ref, np.full((1, n), 2.5, np.float32), 40, 24, pol)
    # signed zeros, negatives, infinities, NaNs of both signs, denormals
    special = np.array([0.0, -0.0, 1e-41, -1e-41, np.inf, -np.inf, 3.0, -3.0], dtype=np.float32)
    E = np.tile(special, n // len(special))[None, :].copy()
    E.view(np.uint32)[0, 9] = 0x7FC00000
    E.view(np.uint32)[0, 17] = 0xFFC00000
    for k in (1, 3, 9, 20, 40, 59):
        check_select(b, ref, E, 0, n, b.Policy(2, k, 2, 0.5))       # undecayed: every bit pattern survives
    check_select(b, ref, E, n, 0, b.Policy(2, 9, 2, 0.5))            # decayed: denormals halve, never flush
    # scores that differ only in the last bit
    base = np.float32(5.0)
    E = np.nextafter(np.full(n, base, np.float32), np.float32(9), dtype=np.float32)
    E[::2] = base
    check_select(b, ref, E[None, :].copy(), 0, n, b.Policy(1, 20, 1, 1.0))


def test_decay_keeps_denormals(b):
    E = np.array([[1e-41, 2e-45, 1.0, 1.0]], dtype=np.float32)
    _, out = gpu_select(b, E, 4, 0, b.Policy(1, 1, 1, 0.5))             # budget 3 < 4: selection path
    want = E * np.float32(0.5)
    assert out[0, 0] == want[0, 0] and out[0, 0] != 0
    _, out = gpu_select(b, E, 4, 0, b.Policy(2, 2, 2, 0.5))             # keep-all path
    np.testing.assert_array_equal(out.view(np.uint32), want.view(np.uint32))


def test_decay_select_is_deterministic(b):
    rng = np.random.default_rng(9)
    E = (rng.integers(0, 9, (2, 5000)) / 4.0).astype(np.float32)
    pol = b.Policy(4, 2000, 300, 0.9)
    first = gpu_select(b, E, 4500, 500, pol)
    for _ in range(20):
        again = gpu_select(b, E, 4500, 500, pol)
        np.testing.assert_array_equal(first[0], again[0])
        np.testing.assert_array_equal(first[1].view(np.uint32), again[1].view(np.uint32))


# ----------------------------------------------------------------------------------- compact
def run_compact(b, ref, k_src, v_src, kept, n_src=None):
    n_streams, n_keep = kept.shape
    shape = k_src.shape[:3] + (n_keep + 2,) + k_src.shape[4:]
    k_dst = torch.full(shape, 77, dtype=k_src.dtype, device=DEV)
    v_dst = None if v_src is None else torch.full(shape, 77, dtype=v_src.dtype, device=DEV)
    kd = torch.from_numpy(kept).to(DEV)
    b.sirllm_compact_kv(k_src, v_src, k_dst, v_dst, kd, n_keep, n_src=n_src)
    torch.cuda.synchronize()
    rk, rv = ref.compact_kv(to_np_strided(k_src), None if v_src is None else to_np_strided(v_src), kept, n_src=n_src)
    gk = to_np(k_dst)
    np.testing.assert_array_equal(gk[:, :, :, :n_keep], rk)
    assert bool((k_dst[:, :, :, n_keep:] == 77).all())                   # slots past n_keep untouched
    if v_src is not None:
        gv = to_np(v_dst)
        np.testing.assert_array_equal(gv[:, :, :, :n_keep], rv)
        assert bool((v_dst[:, :, :, n_keep:] == 77).all())


@pytest.mark.parametrize("S,L,H,P,D,dtype,with_v", [
    (2, 3, 2, 300, 128, torch.bfloat16, True),      # 256-byte rows, three layers
    (1, 40, 2, 70, 64, torch.float32, True),        # more layers than one launch carries in its arguments (32)
    (1, 33, 1, 50, 16, torch.float16, False),       # K only; one head per layer
    (2, 2, 3, 41, 100, torch.bfloat16, True),       # 200-byte rows: 8-byte vectors
    (1, 2, 2, 33, 5, torch.int16, True),            # 10-byte rows: 2-byte vectors
    (1, 4, 8, 2000, 128, torch.bfloat16, True),     # several tiles per plane
    (2, 3, 4, 8192, 128, torch.bfloat16, True),     # 256-byte rows, planes 2 MiB apart, 1.2 MiB kept: tiles exchanged by plane
])
def test_compact_per_layer_tensors_matches_oracle(b, ref, S, L, H, P, D, dtype, with_v):
    """sirllm_compact_kv_layers: the cache as one [streams, heads, slots, head_dim] tensor per layer, sources and
    destinations allocated separately (and destinations as views with padded slots), against the oracle layer by
    layer; slots past n_keep and the padding stay untouched."""
    rng = np.random.default_rng(S * 1000 + L * 10 + D)
    g0 = torch.Generator(device=DEV).manual_seed(L * 7 + D)
    def make(n):
        t = torch.randint(-30000, 30000, (S, H, n, D), generator=g0, device=DEV, dtype=torch.int32)
        return t.to(dtype) if dtype.is_floating_point else t.to(dtype)
    ks = [make(P) for _ in range(L)]
    vs = [make(P) for _ in range(L)] if with_v else None
    n_keep = max(1, int(P * 0.6))
    kept = np.stack([np.sort(rng.choice(P, n_keep, replace=False)) for _ in range(S)]).astype(np.int32)
    kept[0, -1] = P + 5 if P > 40 else kept[0, -1]                   # an index with no source slot: a zero row
    pad = 3
    kd_full = [torch.full((S, H, n_keep + pad, D + 8), 77, dtype=dtype, device=DEV) for _ in range(L)]
    vd_full = [torch.full((S, H, n_keep + pad, D + 8), 77, dtype=dtype, device=DEV) for _ in range(L)] if with_v else None
    kd = [t[:, :, :, :D] for t in kd_full]
    vd = [t[:, :, :, :D] for t in vd_full] if with_v else None
    b.sirllm_compact_kv_layers(ks, vs, kd, vd, torch.from_numpy(kept).to(DEV), n_keep)
    torch.cuda.synchronize()
    for l in range(L):
        rk, rv = ref.compact_kv(to_np(ks[l])[:, None], to_np(vs[l])[:, None] if with_v else None, kept)
        np.testing.assert_array_equal(to_np(kd_full[l])[:, :, :n_keep, :D], rk[:, 0])
        if with_v:
            np.testing.assert_array_equal(to_np(vd_full[l])[:, :, :n_keep, :D], rv[:, 0])
        for full in ([kd_full[l]] + ([vd_full[l]] if with_v else [])):
            assert bool((full[:, :, n_keep:] == 77).all()) and bool((full[:, :, :, D:] == 77).all())


def to_np_strided(t):
    """Host copy of a possibly strided device view, as a contiguous array (the oracle takes any strides itself)."""
    return to_np(t)


@pytest.mark.parametrize("S,L,H,P,D,dtype", [
    (1, 2, 2, 96, 16, torch.float32),       # tiny workload: 64-byte rows
    (2, 3, 2, 300, 128, torch.bfloat16),    # 256-byte rows
    (1, 2, 3, 50, 128, torch.float16),
    (1, 1, 2, 40, 100, torch.bfloat16),     # 200-byte rows: 8-byte vectors
    (1, 1, 2, 40, 6, torch.int16),          # 12-byte rows: 4-byte vectors
    (1, 2, 1, 33, 5, torch.int16),          # 10-byte rows: 2-byte vectors
    (1, 1, 1, 33, 7, torch.uint8),          # 7-byte rows: byte copies
    (1, 1, 2, 20, 24, torch.float64),       # 8-byte elements
    (2, 2, 2, 1000, 64, torch.float32),     # several tiles and a ragged last tile
])
def test_compact_matches_oracle(b, ref, S, L, H, P, D, dtype):
    rng = np.random.default_rng(P * 13 + D)
    tag_k = synth.tagged_kv(S, L, H, P, D, 0)
    tag_v = synth.tagged_kv(S, L, H, P, D, 1)
    if dtype in (torch.uint8,):
        tag_k, tag_v = tag_k % 251, tag_v % 241
    elif dtype in (torch.int16, torch.float16, torch.bfloat16):
        tag_k, tag_v = tag_k % 32749, tag_v % 32719
    k = tag_k.to(dtype).to(DEV)
    v = tag_v.to(dtype).to(DEV)
    n_keep = max(1, (2 * P) // 3)
    kept = np.stack([np.sort(rng.choice(P, n_keep, replace=False)) for _ in range(S)]).astype(np.int32)
    run_compact(b, ref, k, v, kept)
    run_compact(b, ref, k, None, kept[:, : max(1, n_keep // 2)])


@pytest.mark.parametrize("P", [512, 600, 4096], ids=["planes 128 KB apart", "planes 150 KB apart", "planes 1 MB apart"])
@pytest.mark.parametrize("dtype,D", [(torch.bfloat16, 128), (torch.float32, 64), (torch.bfloat16, 256), (torch.float32, 512)],
                         ids=["256-byte rows bf16", "256-byte rows f32", "512-byte rows", "2 KB rows"])
def test_compact_power_of_two_rows(b, ref, P, dtype, D):
    """Rows of 256 bytes, 512 bytes and of 1 KB and more (a power of two) take single-wave tiles: a wave copies four or
    two whole rows, or 64 vectors of one, and fetches its kept indices by scalar loads (clamped at the end of the
    list); where the source planes lie a power of two apart (P = 512, 4096) the tiles of every group of eight are
    exchanged by the plane index once a compacted plane holds 1 MiB, the ragged last group excepted (here: the largest
    kept counts of P = 4096 and of the longer rows).  Kept counts around the edges of a wave's rows and
    of a group of eight tiles, twelve and twenty planes (every value of the plane index modulo 8), lists with runs,
    with entries that have no source slot, K alone and K with V."""
    rng = np.random.default_rng(P + D)
    for S, L, H in ((1, 3, 4), (2, 5, 2)):
        k = (synth.tagged_kv(S, L, H, P, D, 0) % 32749).to(dtype).to(DEV)
        v = (synth.tagged_kv(S, L, H, P, D, 1) % 32719).to(dtype).to(DEV)
        for n_keep in (1, 3, 4, 5, 31, 32, 33, 63, 100, P // 2 + 1, P - 1, P):
            kept = np.stack([np.sort(rng.choice(P, n_keep, replace=False)) for _ in range(S)]).astype(np.int32)
            if n_keep >= 33:
                kept[0, n_keep // 2:] = np.arange(P - (n_keep - n_keep // 2), P)     # a run at the end, like a recent window
                kept[0] = np.sort(kept[0])
                kept[-1, 7] = P + 5                                                   # no such slot: a zero row
            run_compact(b, ref, k, v, kept)
        run_compact(b, ref, k, None, np.stack([np.arange(40, 40 + 77)] * S).astype(np.int32), n_src=100)   # slots >= 100: zero rows


def test_compact_strided_views_and_bad_indices(b, ref):
    big = synth.tagged_kv(2, 2, 3, 40, 24, 0).to(torch.float32).to(DEV)
    k = big[:, :, :2, :30, :16]                       # padded heads, slots and channels
    v = (big * 2)[:, :, :2, :30, :16]
    kept = np.array([[0, 5, 29, 30, -1, 7], [1, 2, 3, 4, 100000, 28]], dtype=np.int32)   # 30, -1, 100000: no such slot
    shape = (2, 2, 2, 9, 16)
    k_dst = torch.full(shape, 77.0, device=DEV)
    v_dst = torch.full(shape, 77.0, device=DEV)
    b.sirllm_compact_kv(k, v, k_dst, v_dst, torch.from_numpy(kept).to(DEV), 6, n_src=30)
    torch.cuda.synchronize()
    rk, rv = ref.compact_kv(to_np(big)[:, :, :2, :30, :16], to_np(big * 2)[:, :, :2, :30, :16], kept, n_src=30)
    np.testing.assert_array_equal(to_np(k_dst)[:, :, :, :6], rk)
    np.testing.assert_array_equal(to_np(v_dst)[:, :, :, :6], rv)
    assert (rk[0, :, :, 3] == 0).all() and (to_np(k_dst)[0, :, :, 4] == 0).all()
    assert (to_np(k_dst)[:, :, :, 6:] == 77).all()


def test_compact_many_planes_and_streams(b, ref):
    # more planes than one grid dimension holds (the launch is cut into slices of 65535 planes)
    rng = np.random.default_rng(5)
    k = torch.from_numpy(rng.integers(0, 2**31 - 1, (1, 260, 260, 5, 4)).astype(np.int32)).to(DEV)
    kept = np.array([[4, 0, 2]], dtype=np.int32)
    run_compact(b, ref, k, k + 1, kept)
    k = torch.from_numpy(rng.integers(0, 2**31 - 1, (70, 2, 1, 6, 4)).astype(np.int32)).to(DEV)
    kept = np.stack([np.sort(rng.choice(6, 4, replace=False)) for _ in range(70)]).astype(np.int32)
    run_compact(b, ref, k, None, kept)


# --------------------------------------------------------------------------------- whole step
def gpu_step(b, w, z, tok, held, k_c, v_c, pol=None):
    """Run sirllm_step on device tensors; returns host copies of everything it wrote."""
    pol = pol or b.Policy(w.n_sink, w.n_topk, w.n_recent, w.decay)
    n_streams, n_held = held.shape
    n_new = z.shape[0] // n_streams
    n_cand = n_held + n_new
    n_keep = min(n_cand, pol.n_sink + pol.n_topk + pol.n_recent)
    E = torch.full((n_streams, n_cand), -5.0, device=DEV)
    E[:, :n_held] = held
    idx = torch.full((n_streams, n_keep), -7, dtype=torch.int32, device=DEV)
    out = torch.full((n_streams, n_keep), -7.0, device=DEV)
    shape = k_c.shape[:3] + (n_keep,) + k_c.shape[4:]
    k_dst = torch.zeros(shape, dtype=k_c.dtype, device=DEV)
    v_dst = torch.zeros(shape, dtype=v_c.dtype, device=DEV)
    got = b.sirllm_step(z, tok, w.vocab, E, n_held, n_new, pol, k_c, v_c, k_dst, v_dst, idx, out)
    torch.cuda.synchronize()
    assert got == n_keep
    return dict(E=E, idx=idx, out=out, k=k_dst, v=v_dst, n_keep=n_keep, evicted=n_cand > n_keep)


def check_step_against_oracle(b, ref, w, z, tok, held, k_c, v_c, g, pol=None):
    """Scores within tolerance; then the oracle's select + gather, fed the GPU's scores, bit for bit."""
    pol = pol or b.Policy(w.n_sink, w.n_topk, w.n_recent, w.decay)
    n_streams, n_held = held.shape
    n_new = z.shape[0] // n_streams
    Eg = to_np(g["E"])
    want = ref.score(to_np(z), to_np(tok), vocab=w.vocab).reshape(n_streams, n_new)
    assert_scores_close(Eg[:, n_held:], want)
    np.testing.assert_array_equal(Eg[:, :n_held].view(np.uint32), to_np(held).view(np.uint32))   # held part untouched
    ri, ro = ref.decay_select(Eg, n_held, n_new, ref.Policy(*pol))
    np.testing.assert_array_equal(to_np(g["idx"]), ri)
    np.testing.assert_array_equal(to_np(g["out"]).view(np.uint32), ro.view(np.uint32))
    if g["evicted"]:
        rk, rv = ref.compact_kv(to_np(k_c), to_np(v_c), ri, n_src=n_held + n_new)
        assert np.array_equal(to_np(g["k"]), rk) and np.array_equal(to_np(g["v"]), rv)
    else:
        assert not to_np(g["k"]).any() and not to_np(g["v"]).any()       # destination untouched


def test_step_tiny_dialogue_four_turns(b, ref):
    w = synth.WORKLOADS["tiny"]
    held = torch.zeros((1, 0), device=DEV)
    shape0 = (1, w.n_layers, w.n_kv_heads, 0, w.head_dim)
    K = torch.zeros(shape0, device=DEV)
    V = torch.zeros(shape0, device=DEV)
    for turn in range(1, w.n_turns + 1):
        z = synth.make_logits(w, turn=turn, device=DEV)
        tok = synth.make_token_ids(w, turn=turn, device=DEV)
        k_c = torch.cat([K, synth.make_kv(w, n_pos=w.n_new, turn=turn, device=DEV, which="k")], dim=3).contiguous()
        v_c = torch.cat([V, synth.make_kv(w, n_pos=w.n_new, turn=turn, device=DEV, which="v")], dim=3).contiguous()
        g = gpu_step(b, w, z, tok, held, k_c, v_c)
        check_step_against_oracle(b, ref, w, z, tok, held, k_c, v_c, g)
        assert g["n_keep"] == w.budget
        held, K, V = g["out"], g["k"], g["v"]


@pytest.mark.parametrize("n_streams,n_held,n_new,pol", [
    (1, 100, 40, (4, 50, 40, 0.9)),     # n_new == n_recent: new tokens never compete
    (1, 100, 40, (4, 80, 8, 0.9)),      # n_new > n_recent: selection depends on this turn's scores
    (3, 60, 30, (4, 30, 10, 0.8)),      # several streams
    (2, 10, 12, (4, 20, 8, 0.9)),       # under budget: nothing evicted
    (2, 90, 0, (4, 20, 8, 0.9)),        # no new tokens: decay + select + compact only
    (1, 0, 50, (4, 20, 8, 0.9)),        # empty cache
])
def test_step_small_shapes(b, ref, n_streams, n_held, n_new, pol):
    w = synth.WORKLOADS["tiny"]
    pol = b.Policy(*pol)
    g0 = torch.Generator(device=DEV).manual_seed(n_held * 100 + n_new)
    z = torch.randn((n_streams * n_new, 777), generator=g0, device=DEV) * 2
    tok = torch.randint(0, 777, (n_streams * n_new,), generator=g0, device=DEV, dtype=torch.int32)
    held = torch.rand((n_streams, n_held), generator=g0, device=DEV) * 6
    k_c = torch.randn((n_streams, 2, 2, n_held + n_new, 16), generator=g0, device=DEV)
    v_c = torch.randn((n_streams, 2, 2, n_held + n_new, 16), generator=g0, device=DEV)
    import dataclasses
    w2 = dataclasses.replace(w, vocab=777)
    g = gpu_step(b, w2, z, tok, held, k_c, v_c, pol=pol)
    check_step_against_oracle(b, ref, w2, z, tok, held, k_c, v_c, g, pol=pol)


@pytest.mark.parametrize("S,L,H,n_held,n_new,pol,D,kv_dt", [
    (2, 4, 4, 2400, 600, (4, 1396, 600, 0.9), 128, torch.bfloat16),     # the recent window is exactly this turn's tokens
    (1, 8, 4, 3000, 500, (4, 1000, 1100, 0.8), 128, torch.bfloat16),    # the window holds held slots as well as the new ones
    (3, 2, 8, 2000, 700, (0, 500, 700, 1.0), 64, torch.float32),        # no sinks, 4-byte elements
    (2, 4, 4, 2400, 600, (4, 1396, 600, 0.9), 120, torch.bfloat16),     # 240-byte rows: 15 vectors, not a power of two
    (2, 4, 4, 2400, 600, (4, 1396, 600, 0.9), 100, torch.bfloat16),     # 200-byte rows: 8-byte vectors
    # 8193..16384 candidate slots with the new tokens inside the recent window: scoring and selection still share a
    # launch, the selecting workgroup with sixteen slots per lane; at 16385 slots they do not any more
    (1, 2, 2, 9000, 1000, (4, 5000, 1500, 0.9), 64, torch.bfloat16),
    (2, 1, 2, 15000, 1384, (4, 8000, 1384, 0.8), 32, torch.float32),
    (1, 1, 2, 15001, 1384, (4, 8000, 1384, 0.8), 32, torch.float32),
])
def test_step_mid_sizes(b, ref, S, L, H, n_held, n_new, pol, D, kv_dt):
    """Whole steps between the small shapes and the benchmark's: a few thousand slots, tens of planes, rows of 256,
    240 and 200 bytes (16-byte vectors with a power-of-two and an odd count per row, 8-byte vectors), self-identifying
    K/V payloads; scoring and selection share a launch (no new token can compete in Top_k) up to 16384 slots."""
    import dataclasses
    V = 2000
    w2 = dataclasses.replace(synth.WORKLOADS["tiny"], vocab=V)
    pol = b.Policy(*pol)
    g0 = torch.Generator(device=DEV).manual_seed(n_held + D)
    z = (torch.randn((S * n_new, V), generator=g0, device=DEV) * 3).to(torch.bfloat16)
    tok = torch.randint(0, V, (S * n_new,), generator=g0, device=DEV, dtype=torch.int32)
    held = torch.rand((S, n_held), generator=g0, device=DEV) * 6
    n_cand = n_held + n_new
    k_c = (synth.tagged_kv(S, L, H, n_cand, D, 0) % 32749).to(kv_dt).to(DEV)
    v_c = (synth.tagged_kv(S, L, H, n_cand, D, 1) % 32719).to(kv_dt).to(DEV)
    g = gpu_step(b, w2, z, tok, held, k_c, v_c, pol=pol)
    check_step_against_oracle(b, ref, w2, z, tok, held, k_c, v_c, g, pol=pol)


# ------------------------------------------------------------------------- baseline policies
BASELINE_CASES = [
    # n_streams, n_cand, n_sink, k, n_recent
    (2, 50, 4, 10, 6), (1, 26, 4, 5, 2), (1, 29, 4, 5, 2), (1, 20, 2, 8, 3), (3, 1078, 4, 1020, 0),
    (2, 600, 4, 100, 16), (1, 4096, 4, 1532, 512), (2, 8192, 4, 3068, 1024), (1, 32768, 4, 16000, 68),
    (2, 30, 4, 20, 8), (1, 40, 0, 7, 0), (1, 40, 4, 0, 6), (1, 5000, 0, 1, 0), (1, 5000, 3, 4996, 0),
    # the random policy's workgroup keeps 1, 4, 8, 16 or 32 slots per thread: 8193..16384 slots reach the 16-slot
    # instance, 16385..32768 the 32-slot one
    (1, 8193, 4, 4000, 193), (2, 12000, 4, 6000, 500), (1, 16384, 4, 1, 0), (2, 12345, 0, 12000, 45),
    (1, 16385, 4, 8000, 384), (2, 26000, 4, 13000, 1000),
    # above 32768 slots per stream the random policy goes through the multi-workgroup selection (tiles of 8192 slots):
    # one slot past the limit, a ragged last tile, several streams, a 128K-slot cache, all-but-one and one kept
    (1, 32769, 4, 16000, 68), (3, 40000, 4, 20000, 1000), (2, 133120, 4, 129020, 2048), (1, 50000, 0, 49999, 0),
    (2, 70001, 4, 1, 0), (1, 65536, 4, 0, 100),
]


@pytest.mark.parametrize("kind", [0, 1, 2])
@pytest.mark.parametrize("case", BASELINE_CASES, ids=[str(c) for c in BASELINE_CASES])
def test_baseline_select_matches_oracle(b, ref, kind, case):
    n_streams, n_cand, n_sink, k, n_recent = case
    pol = b.Policy(n_sink, k, n_recent, 0.0)
    seed, turn = (7 << 32) | 12345, (3 << 32) | 99
    want = ref.baseline_select(kind, n_streams, n_cand, ref.Policy(*pol), seed=seed, turn=turn)
    n_keep = want.shape[1]
    idx = torch.full((n_streams, n_keep + 3), -7, dtype=torch.int32, device=DEV)
    # scratch is asked for above 32768 slots only; it arrives dirty, the call clears what it uses
    nbytes = b.sirllm_workspace_bytes(n_streams, n_cand, 0, 0)
    assert (nbytes > 0) == (n_cand > 32768)
    ws = torch.full((nbytes,), 0x5a, dtype=torch.uint8, device=DEV) if nbytes else None
    got_keep = b.sirllm_baseline_select(kind, n_cand, pol, idx, seed=seed, turn=turn, workspace=ws)
    torch.cuda.synchronize()
    assert got_keep == n_keep
    got = to_np(idx)
    np.testing.assert_array_equal(got[:, :n_keep], want)
    assert (got[:, n_keep:] == -7).all()


def test_baseline_policies_feed_the_same_compaction(b, ref):
    # a baseline's kept list goes through sirllm_compact_kv like the entropy policy's
    S, L, H, P, D = 2, 2, 2, 200, 32
    k = synth.tagged_kv(S, L, H, P, D, 0).to(torch.float32).to(DEV)
    v = synth.tagged_kv(S, L, H, P, D, 1).to(torch.float32).to(DEV)
    pol = b.Policy(4, 60, 16, 0.0)
    for kind in (0, 1, 2):
        idx = torch.zeros((S, 80), dtype=torch.int32, device=DEV)
        n_keep = b.sirllm_baseline_select(kind, P, pol, idx, seed=5, turn=kind)
        torch.cuda.synchronize()
        kept = to_np(idx)[:, :n_keep]
        np.testing.assert_array_equal(kept, ref.baseline_select(kind, S, P, ref.Policy(*pol), seed=5, turn=kind))
        run_compact(b, ref, k, v, kept)


# --------------------------------------------------------------------- randomised whole steps
def test_step_random_shapes(b, ref):
    """Sixty seeded random shapes through sirllm_step: stream counts, cache fill, policy sizes, vocabulary
    lengths, row padding, logits dtype, K/V element size and head_dim all vary together."""
    import dataclasses
    rng = np.random.default_rng(2024)
    base = synth.WORKLOADS["tiny"]
    for case in range(60):
        S = int(rng.integers(1, 4))
        n_held = int(rng.integers(0, 300))
        n_new = int(rng.integers(0, 90))
        if n_held + n_new == 0:
            n_new = 1
        n_sink = int(rng.integers(0, 6))
        k = int(rng.integers(0, 200))
        n_recent = int(rng.integers(0, 100))
        V = int(rng.integers(1, 3000))
        ld = V + int(rng.integers(0, 9))
        dt = torch.bfloat16 if rng.integers(2) else torch.float32
        kv_dt = [torch.float32, torch.bfloat16, torch.uint8][int(rng.integers(3))]
        D = int(rng.choice([8, 16, 24, 64, 128]))
        L, H = int(rng.integers(1, 3)), int(rng.integers(1, 4))
        pol = b.Policy(n_sink, k, n_recent, float(rng.choice([1.0, 0.9, 0.5])))
        g0 = torch.Generator(device=DEV).manual_seed(case)
        z = (torch.randn((S * n_new, ld), generator=g0, device=DEV) * 3).to(dt)
        if ld > V and n_new:
            z[:, V:] = 1.0e4
        tok = torch.randint(0, V, (S * n_new,), generator=g0, device=DEV, dtype=torch.int32)
        levels = int(rng.choice([4, 1000000]))
        held = (torch.randint(0, levels, (S, n_held), generator=g0, device=DEV) / 7.0).to(torch.float32)
        n_cand = n_held + n_new
        if kv_dt == torch.uint8:
            k_c = torch.randint(0, 255, (S, L, H, n_cand, D), generator=g0, device=DEV, dtype=torch.uint8)
            v_c = torch.randint(0, 255, (S, L, H, n_cand, D), generator=g0, device=DEV, dtype=torch.uint8)
        else:
            k_c = torch.randn((S, L, H, n_cand, D), generator=g0, device=DEV).to(kv_dt)
            v_c = torch.randn((S, L, H, n_cand, D), generator=g0, device=DEV).to(kv_dt)
        w2 = dataclasses.replace(base, vocab=V)
        print(f"case {case}: S={S} held={n_held} new={n_new} pol={tuple(pol)} V={V} ld={ld} {dt} kv={kv_dt} D={D}", flush=True)
        try:
            g = gpu_step(b, w2, z, tok, held, k_c, v_c, pol=pol)
            check_step_against_oracle(b, ref, w2, z, tok, held, k_c, v_c, g, pol=pol)
        except AssertionError as e:
            raise AssertionError(f"case {case}: {e}") from e


# ------------------------------------------------------------------------ in-place compaction
def inplace_scratch(b, dirty=0x5A):
    """A workspace for the in-place compaction's ticket counter (dirty on purpose: the call clears it itself)."""
    return torch.full((b.SIRLLM_INPLACE_WORKSPACE_BYTES,), dirty, dtype=torch.uint8, device=DEV)


@pytest.mark.parametrize("ticket", [False, True], ids=["by block index", "by ticket"])
@pytest.mark.parametrize("S,L,H,P,D,dtype,frac", [
    (1, 2, 2, 96, 16, torch.float32, 0.33),
    (2, 3, 2, 300, 128, torch.bfloat16, 0.6),
    (1, 1, 2, 40, 100, torch.bfloat16, 0.5),      # 8-byte vectors
    (1, 2, 1, 33, 5, torch.int16, 0.7),           # 2-byte vectors
    (1, 1, 1, 33, 7, torch.uint8, 0.5),
    (2, 2, 2, 5000, 64, torch.float32, 0.5),      # many chunks per plane
    (1, 2, 2, 4096, 128, torch.bfloat16, 0.97),   # almost everything kept: short moves
    (1, 2, 2, 1078, 128, torch.bfloat16, 0.95),
    (4, 32, 32, 40, 8, torch.int16, 0.6),         # 8192 planes: from here on a workspace switches the ticket order on
    (3, 48, 32, 70, 64, torch.bfloat16, 0.8),     # 9216 planes of 128-byte rows
])
def test_compact_inplace_matches_oracle(b, ref, S, L, H, P, D, dtype, frac, ticket):
    """Without a workspace the workgroups take their planes by block index, with one by ticket."""
    rng = np.random.default_rng(P * 7 + D)
    mod = 251 if dtype == torch.uint8 else (32749 if dtype in (torch.int16, torch.bfloat16) else 1 << 31)
    k = (synth.tagged_kv(S, L, H, P, D, 0) % mod).to(dtype).to(DEV)
    v = (synth.tagged_kv(S, L, H, P, D, 1) % mod).to(dtype).to(DEV)
    n_keep = max(1, int(P * frac))
    kept = np.stack([np.sort(rng.choice(P, n_keep, replace=False)) for _ in range(S)]).astype(np.int32)
    kept[0, :min(4, n_keep)] = np.arange(min(4, n_keep))       # sinks stay put
    kept = np.sort(kept, axis=1)
    if len(np.unique(kept[0])) != n_keep:
        kept[0] = np.sort(rng.choice(P, n_keep, replace=False))
    hk, hv = to_np(k).copy(), to_np(v).copy()
    ref.compact_kv_inplace(hk, hv, kept)
    ws = inplace_scratch(b) if ticket else None
    b.sirllm_compact_kv_inplace(k, v, torch.from_numpy(kept).to(DEV), n_keep, workspace=ws)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(k), hk), "K differs (kept rows or the untouched tail)"
    assert np.array_equal(to_np(v), hv), "V differs"
    # shifts by one: every row is the source of its left neighbour
    k2 = (synth.tagged_kv(S, L, H, P, D, 0) % mod).to(dtype).to(DEV)
    chain = np.arange(1, P, dtype=np.int32)[None, :].repeat(S, 0)
    h2 = to_np(k2).copy()
    ref.compact_kv_inplace(h2, None, chain)
    ws = inplace_scratch(b) if ticket else None
    b.sirllm_compact_kv_inplace(k2, None, torch.from_numpy(chain).to(DEV), P - 1, workspace=ws)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(k2), h2)


@pytest.mark.parametrize("ticket", [False, True], ids=["by block index", "by ticket"])
@pytest.mark.parametrize("S,L,H,P,D,dtype,frac,with_v", [
    (2, 3, 2, 300, 128, torch.bfloat16, 0.6, True),
    (1, 40, 2, 5000, 64, torch.float32, 0.5, True),     # more layers than one launch carries (32); many chunks per plane
    (1, 33, 1, 50, 16, torch.float16, 0.9, False),      # K only, one head per layer
    (1, 2, 2, 33, 5, torch.int16, 0.7, True),           # 2-byte vectors
    (2, 34, 64, 40, 8, torch.int16, 0.6, True),         # 8704 planes: ticket order with a workspace
])
def test_compact_inplace_per_layer_tensors_matches_oracle(b, ref, S, L, H, P, D, dtype, frac, with_v, ticket):
    """sirllm_compact_kv_inplace_layers: one [streams, heads, slots, head_dim] tensor per layer, compacted in place,
    against the oracle's in-place compaction layer by layer (kept rows and the untouched tail alike)."""
    rng = np.random.default_rng(P * 11 + D + L)
    mod = 32749 if dtype in (torch.int16, torch.bfloat16, torch.float16) else 1 << 31
    k = [(synth.tagged_kv(S, 1, H, P, D, 2 * l) % mod).to(dtype)[:, 0].contiguous().to(DEV) for l in range(L)]
    v = [(synth.tagged_kv(S, 1, H, P, D, 2 * l + 1) % mod).to(dtype)[:, 0].contiguous().to(DEV) for l in range(L)] if with_v else None
    n_keep = max(1, int(P * frac))
    kept = np.stack([np.sort(rng.choice(P, n_keep, replace=False)) for _ in range(S)]).astype(np.int32)
    want_k = [to_np(t)[:, None].copy() for t in k]
    want_v = [to_np(t)[:, None].copy() for t in v] if with_v else None
    for l in range(L):
        ref.compact_kv_inplace(want_k[l], want_v[l] if with_v else None, kept)
    ws = inplace_scratch(b) if ticket else None
    b.sirllm_compact_kv_inplace_layers(k, v, torch.from_numpy(kept).to(DEV), n_keep, workspace=ws)
    torch.cuda.synchronize()
    for l in range(L):
        assert np.array_equal(to_np(k[l]), want_k[l][:, 0]), f"layer {l}: K differs"
        if with_v:
            assert np.array_equal(to_np(v[l]), want_v[l][:, 0]), f"layer {l}: V differs"


@pytest.mark.parametrize("ticket", [False, True], ids=["by block index", "by ticket"])
@pytest.mark.parametrize("dtype,D", [(torch.float32, 4), (torch.int16, 4), (torch.int16, 2), (torch.int16, 1), (torch.uint8, 1),
                                     (torch.bfloat16, 128)])
def test_compact_inplace_chunk_boundaries(b, ref, dtype, D, ticket):
    """Planes of 1, CH - 1, CH, CH + 1 and 2 CH + 1 vectors for every vector width the kernels use (16, 8, 4, 2, 1
    bytes), at the default launch shape: CH = 4096 vectors is one chunk of the walk, whose counted wait must also
    hold when a chunk is ragged or the look-ahead chunk lies wholly past the end of the plane."""
    row_vecs = 16 if D == 128 else 1                                  # vectors per row: rows of 256 bytes, else one vector
    for ch in (4096,):
        for n_vec in (1, ch - 1, ch, ch + 1, 2 * ch - 1, 2 * ch, 2 * ch + 1, 3 * ch + 1):
            n_keep = max(1, n_vec // row_vecs)
            P = n_keep + 1 + n_keep // 3
            rng = np.random.default_rng(n_vec + D)
            mod = 251 if dtype == torch.uint8 else (32749 if dtype in (torch.int16, torch.bfloat16) else 1 << 31)
            k = (synth.tagged_kv(1, 1, 2, P, D, 0) % mod).to(dtype).to(DEV)
            kept = np.sort(rng.choice(P, n_keep, replace=False)).astype(np.int32)[None, :]
            hk = to_np(k).copy()
            ref.compact_kv_inplace(hk, None, kept)
            ws = inplace_scratch(b) if ticket else None
            b.sirllm_compact_kv_inplace(k, None, torch.from_numpy(kept).to(DEV), n_keep, workspace=ws)
            torch.cuda.synchronize()
            assert np.array_equal(to_np(k), hk), f"{n_vec} vectors of {k.element_size() * D} bytes"


@pytest.mark.parametrize("order", ["SLPHD", "SPLHD", "SLPHD_padded", "SLHPD"])
@pytest.mark.parametrize("dtype,D", [(torch.bfloat16, 128), (torch.float32, 16), (torch.int16, 5)])
def test_compact_slot_major_layouts(b, ref, order, dtype, D):
    """Caches stored slot-major -- [slot][head][dim] per layer, or [slot][layer][head][dim] -- handed over as
    strided [stream][layer][head][slot][dim] views: heads (and layers) that lie back to back are copied as one
    longer row, and the result is the same as for any other strides.  Out of place and in place."""
    S, L, H, P, n_keep = 2, 3, 4, 700, 333
    rng = np.random.default_rng(P + D)
    mod = 32749 if dtype in (torch.int16, torch.bfloat16) else 1 << 31

    def store(t):            # [S, L, H, P', D] values -> the same values in the layout under test, viewed as [S, L, H, P', D]
        t = t.to(DEV)
        if order == "SLPHD":
            return t.permute(0, 1, 3, 2, 4).contiguous().permute(0, 1, 3, 2, 4)
        if order == "SPLHD":
            return t.permute(0, 3, 1, 2, 4).contiguous().permute(0, 2, 3, 1, 4)
        if order == "SLPHD_padded":     # heads back to back, but a gap after every slot
            buf = torch.zeros((t.shape[0], L, t.shape[3], H + 1, D), dtype=t.dtype, device=DEV)
            buf[:, :, :, :H] = t.permute(0, 1, 3, 2, 4)
            return buf[:, :, :, :H].permute(0, 1, 3, 2, 4)
        return t.contiguous()

    k = store((synth.tagged_kv(S, L, H, P, D, 0) % mod).to(dtype))
    v = store((synth.tagged_kv(S, L, H, P, D, 1) % mod).to(dtype))
    kept = np.stack([np.sort(rng.choice(P, n_keep, replace=False)) for _ in range(S)]).astype(np.int32)
    kept[1, 5] = P + 3                                               # no such slot: a zero row in every head and layer
    kd = store(torch.full((S, L, H, n_keep + 2, D), 77, dtype=dtype))
    vd = store(torch.full((S, L, H, n_keep + 2, D), 77, dtype=dtype))
    b.sirllm_compact_kv(k, v, kd, vd, torch.from_numpy(kept).to(DEV), n_keep)
    torch.cuda.synchronize()
    rk, rv = ref.compact_kv(to_np(k), to_np(v), kept)
    assert np.array_equal(to_np(kd)[:, :, :, :n_keep], rk) and np.array_equal(to_np(vd)[:, :, :, :n_keep], rv)
    assert bool((kd[:, :, :, n_keep:] == 77).all()) and bool((vd[:, :, :, n_keep:] == 77).all())
    kept[1] = np.sort(rng.choice(P, n_keep, replace=False))          # in place needs a strictly ascending list
    hk, hv = to_np(k).copy(), to_np(v).copy()
    ref.compact_kv_inplace(hk, hv, kept)
    b.sirllm_compact_kv_inplace(k, v, torch.from_numpy(kept).to(DEV), n_keep, workspace=inplace_scratch(b))
    torch.cuda.synchronize()
    assert np.array_equal(to_np(k), hk) and np.array_equal(to_np(v), hv)


@pytest.mark.parametrize("ticket", [False, True], ids=["by block index", "by ticket"])
def test_compact_inplace_with_unusable_lists(b, ref, ticket):
    """Lists the header calls unspecified -- not ascending, repeated entries, entries with no source slot -- must
    still leave everything outside the first n_keep slots alone."""
    S, L, H, P, D = 1, 1, 2, 20000, 128
    rng = np.random.default_rng(3)
    n_keep = 15000
    for kind in ("shuffled", "all the same", "descending", "mostly out of range"):
        k = (synth.tagged_kv(S, L, H, P, D, 0) % 32749).to(torch.bfloat16).to(DEV)
        before = to_np(k).copy()
        if kind == "shuffled":
            kept = rng.permutation(P)[:n_keep]
        elif kind == "all the same":
            kept = np.full(n_keep, P - 1)
        elif kind == "descending":
            kept = np.arange(P - 1, P - 1 - n_keep, -1)
        else:
            kept = np.sort(rng.choice(P, n_keep, replace=False))
            kept[::3] = 2 ** 31 - 5
        kept = kept.astype(np.int32)[None, :]
        ws = inplace_scratch(b) if ticket else None
        b.sirllm_compact_kv_inplace(k, None, torch.from_numpy(kept).to(DEV), n_keep, workspace=ws)
        torch.cuda.synchronize()
        after = to_np(k)
        assert np.array_equal(after[:, :, :, n_keep:], before[:, :, :, n_keep:]), kind     # the tail is never written


def test_compact_inplace_strided_view_and_bad_indices(b, ref):
    big = synth.tagged_kv(2, 2, 3, 40, 24, 0).to(torch.float32).to(DEV)
    host = to_np(big).copy()
    view = big[:, :, :2, :30, :16]
    kept = np.array([[0, 5, 29, 30, 31, 35], [1, 2, 3, 4, 100000, 100001]], dtype=np.int32)   # last ones: no such slot
    ref.compact_kv_inplace(host[:, :, :2, :30, :16], None, kept, n_src=30)
    b.sirllm_compact_kv_inplace(view, None, torch.from_numpy(kept).to(DEV), 6, n_src=30)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(big), host)                    # padding heads / slots / channels untouched too


# ------------------------------------------------------------------------------ ragged batches
def run_ragged(b, ref, rng, S, pol, V, dt, n_held, n_new, L=2, H=2, D=16, kv_dt=torch.float32, cap=None,
               tight_new=True, new_cap=None, lmhead_d=None, out_of_place=False):
    """One ragged step on the GPU and in the oracle; compares everything the step writes.  cap / new_cap: the
    bounds on n_cand[s] / n_new[s] promised to the library when they are lower than what the streams hold; a
    stream beyond either, or with a negative n_held, must come back flagged with nothing of its kept list or
    K/V touched.  lmhead_d: the scores come from hidden states of that width and an output embedding matrix
    (sirllm_step_lmhead_ragged) instead of stored logits.  out_of_place: sirllm_step_ragged_out_of_place -- every accepted
    stream's kept slots land in a second pair of buffers (compacted when over budget, as they are otherwise), which must
    keep their sentinel past n_keep and for flagged streams; no source byte may change."""
    n_held, n_new = np.asarray(n_held), np.asarray(n_new)
    n_cand = n_held + n_new
    max_cand = int(n_cand.max()) if cap is None else cap
    budget = pol.n_sink + pol.n_topk + pol.n_recent
    total = int(n_new.sum())
    g0 = torch.Generator(device=DEV).manual_seed(int(rng.integers(1 << 30)))
    if lmhead_d is None:
        z = (torch.randn((total, V + 3), generator=g0, device=DEV) * 3).to(dt)
        if total:
            z[:, V:] = 1.0e4
    else:
        hid = (torch.randn((total, lmhead_d + 8), generator=g0, device=DEV) + 0.5).to(dt)[:, :lmhead_d]
        emb = (torch.randn((V + 2, lmhead_d), generator=g0, device=DEV) * (3.0 / lmhead_d ** 0.5)).to(dt)
    tok = torch.randint(0, V, (total,), generator=g0, device=DEV, dtype=torch.int32)
    scores = torch.full((S, max_cand + 2), -3.0, device=DEV)
    for s in range(S):
        fill = max(0, min(int(n_held[s]), max_cand + 2))  # a stream beyond the promised bound only fills what exists
        scores[s, :fill] = torch.randint(0, 50, (fill,), generator=g0, device=DEV) / 7.0
    k = torch.randn((S, L, H, max_cand + 1, D), generator=g0, device=DEV).to(kv_dt)
    v = torch.randn((S, L, H, max_cand + 1, D), generator=g0, device=DEV).to(kv_dt)
    keep_cap = min(max_cand, budget)
    kept = torch.full((S, keep_cap + 1), -7, dtype=torch.int32, device=DEV)
    out = torch.full((S, keep_cap + 1), -7.0, device=DEV)
    n_keep_dev = torch.full((S,), -9, dtype=torch.int32, device=DEV)
    held_dev = torch.from_numpy(n_held.astype(np.int32)).to(DEV)
    cu = torch.from_numpy(np.concatenate([[0], np.cumsum(n_new)]).astype(np.int32)).to(DEV)
    hs, hk, hv = to_np(scores).copy(), to_np(k).copy(), to_np(v).copy()
    ws = inplace_scratch(b) if rng.integers(2) else None
    if max_cand > 32768:        # the multi-workgroup selection's scratch is required there; it arrives dirty
        ws = torch.full((b.sirllm_workspace_bytes(S, max_cand, 0, 0),), 0x5a, dtype=torch.uint8, device=DEV)
    max_new = min(int(n_new.max()), max_cand) if tight_new else None
    if new_cap is not None:
        max_new = new_cap
    bound_new = max_new if max_new is not None else min(total, max_cand)
    fits_all = (n_held >= 0) & (n_new <= bound_new) & (n_cand <= max_cand)
    if out_of_place:
        kd = torch.full((S, L, H, keep_cap + 1, D), 77, dtype=kv_dt, device=DEV)
        vd = torch.full((S, L, H, keep_cap + 1, D), 77, dtype=kv_dt, device=DEV)
    if out_of_place and lmhead_d is not None:
        ws = torch.full((b.sirllm_step_lmhead_ragged_workspace_bytes(S, max_cand, total, V),), 0x5a, dtype=torch.uint8,
                        device=DEV)
        b.sirllm_step_lmhead_ragged_out_of_place(hid, emb, tok, scores, held_dev, cu, total, max_cand, pol, k, v, kd, vd,
                                                 kept, out, n_keep_dev, ws, max_new=max_new, vocab=V)
    elif out_of_place:
        b.sirllm_step_ragged_out_of_place(z, tok, V, scores, held_dev, cu, total, max_cand, pol, k, v, kd, vd, kept, out,
                                          n_keep_dev, max_new=max_new, workspace=ws)
    elif lmhead_d is None:
        b.sirllm_step_ragged(z, tok, V, scores, held_dev, cu, total, max_cand, pol, k, v, kept, out, n_keep_dev,
                             max_new=max_new, workspace=ws)
    else:
        ws = torch.full((b.sirllm_step_lmhead_ragged_workspace_bytes(S, max_cand, total, V),), 0x5a, dtype=torch.uint8,
                        device=DEV)
        b.sirllm_step_lmhead_ragged(hid, emb, tok, scores, held_dev, cu, total, max_cand, pol, k, v, kept, out,
                                    n_keep_dev, ws, max_new=max_new, vocab=V)
    torch.cuda.synchronize()
    gs, gkeep = to_np(scores), to_np(n_keep_dev)
    # scores: tolerance; then teacher-force the oracle with the GPU's scores for everything exact
    want_scores = hs.copy()
    if total:
        e = ref.score(to_np(z), to_np(tok), vocab=V) if lmhead_d is None else \
            ref.lmhead_score(np.ascontiguousarray(to_np(hid)), to_np(emb)[:V], to_np(tok))
        r0 = 0
        for s in range(S):
            if fits_all[s]:
                want_scores[s, n_held[s]:n_cand[s]] = e[r0:r0 + n_new[s]]
            r0 += n_new[s]
    for s in range(S):
        if not fits_all[s]:
            assert gkeep[s] == -1                             # flagged ...
            assert (to_np(kept)[s] == -7).all()               # ... and its kept list left alone (K/V: compared below)
            if n_cand[s] > max_cand and n_held[s] >= max_cand + 2:
                np.testing.assert_array_equal(gs[s], hs[s])   # no place for its new scores: nothing written at all
            else:
                np.testing.assert_array_equal(gs[s, :max(0, n_held[s])], hs[s, :max(0, n_held[s])])   # held scores intact
            continue
        assert_scores_close(gs[s, n_held[s]:n_cand[s]], want_scores[s, n_held[s]:n_cand[s]],
                            atol=1e-6 if lmhead_d is None else 2e-5)
        np.testing.assert_array_equal(gs[s, :n_held[s]], hs[s, :n_held[s]])
        np.testing.assert_array_equal(gs[s, n_cand[s]:], hs[s, n_cand[s]:])
    ok = [s for s in range(S) if fits_all[s]]
    forced = gs.copy()
    if out_of_place:
        want_kd, want_vd = to_np(torch.full_like(kd, 77)), to_np(torch.full_like(vd, 77))
    # the oracle recomputes the new scores itself; overwrite them with the GPU's afterwards by calling the pieces
    for s in ok:
        h, n = int(n_held[s]), int(n_new[s])
        if h + n == 0:
            assert gkeep[s] == 0
            continue
        ki, so = ref.decay_select(forced[s:s + 1, :h + n], h, n, ref.Policy(*pol))
        assert gkeep[s] == ki.shape[1]
        np.testing.assert_array_equal(to_np(kept)[s, :ki.shape[1]], ki[0])
        np.testing.assert_array_equal(to_np(out)[s, :ki.shape[1]].view(np.uint32), so[0].view(np.uint32))
        assert (to_np(kept)[s, ki.shape[1]:] == -7).all()
        if out_of_place:                                  # every accepted stream moves: compacted, or as it is
            rk, rv = ref.compact_kv(hk[s:s + 1], hv[s:s + 1], ki, n_src=h + n)
            want_kd[s, :, :, :ki.shape[1]], want_vd[s, :, :, :ki.shape[1]] = rk[0], rv[0]
        elif h + n > budget:
            ref.compact_kv_inplace(hk[s:s + 1], hv[s:s + 1], ki, n_src=h + n)
    assert np.array_equal(to_np(k), hk), "K differs (compacted streams, untouched streams or tails)"
    assert np.array_equal(to_np(v), hv), "V differs"
    if out_of_place:
        assert np.array_equal(to_np(kd), want_kd), "destination K differs (compacted streams, or written where nothing may be)"
        assert np.array_equal(to_np(vd), want_vd), "destination V differs"


def test_step_ragged_matches_oracle(b, ref):
    rng = np.random.default_rng(77)
    pol = b.Policy(4, 20, 8, 0.9)                       # budget 32
    # streams under, at and over the budget; empty streams; streams without new tokens
    run_ragged(b, ref, rng, 6, pol, 500, torch.float32, [0, 10, 24, 40, 90, 0], [5, 22, 8, 0, 17, 0])
    run_ragged(b, ref, rng, 3, pol, 777, torch.bfloat16, [100, 31, 0], [1, 1, 64], kv_dt=torch.bfloat16, D=128)
    run_ragged(b, ref, rng, 1, pol, 64, torch.float32, [200], [0])
    run_ragged(b, ref, rng, 4, b.Policy(4, 1020, 0, 0.8), 300, torch.bfloat16, [1024, 1000, 500, 1024], [54, 54, 54, 1],
               L=1, H=2, D=64, kv_dt=torch.bfloat16)
    # a stream larger than the promised bound is flagged and left alone
    run_ragged(b, ref, rng, 3, pol, 100, torch.float32, [10, 60, 20], [5, 30, 5], cap=40, tight_new=False)
    # so is a stream with more new tokens than promised, or with a negative slot count, although each has more
    # slots than the budget and fewer than the bound (its K/V must not be compacted from a stale kept list);
    # with the tight bound scoring and selection share a launch, with the loose one they do not
    run_ragged(b, ref, rng, 4, pol, 100, torch.float32, [40, 30, 50, 45], [5, 20, 8, 3], new_cap=8)
    run_ragged(b, ref, rng, 4, pol, 100, torch.float32, [40, 30, 50, 45], [5, 20, 8, 3], new_cap=12)
    run_ragged(b, ref, rng, 4, pol, 100, torch.bfloat16, [40, -3, 50, -40], [5, 60, 8, 90], cap=100, new_cap=90)
    run_ragged(b, ref, rng, 3, b.Policy(4, 20, 64, 0.9), 100, torch.float32, [90, -3, 100], [5, 60, 8], cap=200, new_cap=64)
    # every stream's new tokens fit the recent window: scoring and selection share a launch
    run_ragged(b, ref, rng, 5, pol, 300, torch.float32, [0, 30, 24, 100, 3], [8, 2, 8, 7, 0])
    run_ragged(b, ref, rng, 3, b.Policy(4, 3068, 1024, 0.85), 2000, torch.bfloat16, [7168, 100, 4000], [1024, 1000, 96],
               L=1, H=2, D=64, kv_dt=torch.bfloat16)
    # the same shapes with a loose bound on the new tokens: three launches
    run_ragged(b, ref, rng, 5, pol, 300, torch.float32, [0, 30, 24, 100, 3], [8, 2, 8, 7, 0], tight_new=False)
    # 5 x 32 x 32 x 2 = 10240 planes: with a workspace the compaction takes its planes by ticket (one stream under
    # budget and one flagged among them: their workgroups draw tickets too and return)
    for _ in range(2):
        run_ragged(b, ref, rng, 5, pol, 200, torch.bfloat16, [40, 10, 90, 33, 60], [8, 5, 3, 8, 20], L=32, H=32, D=8,
                   kv_dt=torch.bfloat16, new_cap=8)
    for _ in range(10):
        S = int(rng.integers(1, 9))
        run_ragged(b, ref, rng, S, b.Policy(int(rng.integers(0, 5)), int(rng.integers(0, 60)), int(rng.integers(0, 20)), 0.7),
                   int(rng.integers(2, 900)), torch.float32 if rng.integers(2) else torch.bfloat16,
                   rng.integers(0, 150, S), rng.integers(0, 40, S))


def test_step_ragged_out_of_place_matches_oracle(b, ref):
    """sirllm_step_ragged_out_of_place against the oracle stream by stream: every accepted stream's kept slots arrive
    in the second pair of buffers, compacted when over budget and as they are otherwise (rows of 64 and 10 bytes: the
    general kernel; of 256 bytes, 512 bytes and 2 KB: the single-wave tiles), flagged streams and everything past a
    stream's n_keep keep the sentinel, no source byte changes; streams under budget, empty streams, fused and
    three-launch selection, a selection over several workgroups."""
    rng = np.random.default_rng(78)
    pol = b.Policy(4, 20, 8, 0.9)                       # budget 32
    run_ragged(b, ref, rng, 6, pol, 500, torch.float32, [0, 10, 24, 40, 90, 0], [5, 22, 8, 0, 17, 0], out_of_place=True)
    run_ragged(b, ref, rng, 3, pol, 777, torch.bfloat16, [100, 31, 0], [1, 1, 64], kv_dt=torch.bfloat16, D=128, out_of_place=True)
    run_ragged(b, ref, rng, 3, pol, 300, torch.bfloat16, [100, 31, 60], [1, 1, 7], kv_dt=torch.bfloat16, D=256, out_of_place=True)
    run_ragged(b, ref, rng, 3, pol, 300, torch.float32, [100, 31, 60], [1, 1, 7], kv_dt=torch.float32, D=512, out_of_place=True)
    run_ragged(b, ref, rng, 2, pol, 300, torch.float32, [100, 31], [1, 1], kv_dt=torch.int16, D=5, out_of_place=True)
    run_ragged(b, ref, rng, 1, pol, 64, torch.float32, [200], [0], out_of_place=True)
    run_ragged(b, ref, rng, 4, b.Policy(4, 1020, 0, 0.8), 300, torch.bfloat16, [1024, 1000, 500, 1024], [54, 54, 54, 1],
               L=1, H=2, D=64, kv_dt=torch.bfloat16, out_of_place=True)
    run_ragged(b, ref, rng, 3, pol, 100, torch.float32, [10, 60, 20], [5, 30, 5], cap=40, tight_new=False, out_of_place=True)
    run_ragged(b, ref, rng, 4, pol, 100, torch.float32, [40, 30, 50, 45], [5, 20, 8, 3], new_cap=8, out_of_place=True)
    run_ragged(b, ref, rng, 4, pol, 100, torch.bfloat16, [40, -3, 50, -40], [5, 60, 8, 90], cap=100, new_cap=90, out_of_place=True)
    run_ragged(b, ref, rng, 3, b.Policy(4, 3068, 1024, 0.85), 2000, torch.bfloat16, [7168, 100, 4000], [1024, 1000, 96],
               L=2, H=4, D=128, kv_dt=torch.bfloat16, out_of_place=True)
    run_ragged(b, ref, rng, 2, b.Policy(4, 30000, 2000, 0.9), 50, torch.float32, [39000, 500], [1000, 20], L=1, H=1, D=8,
               out_of_place=True)
    for _ in range(10):
        S = int(rng.integers(1, 9))
        run_ragged(b, ref, rng, S, b.Policy(int(rng.integers(0, 5)), int(rng.integers(0, 60)), int(rng.integers(0, 20)), 0.7),
                   int(rng.integers(2, 900)), torch.float32 if rng.integers(2) else torch.bfloat16,
                   rng.integers(0, 150, S), rng.integers(0, 40, S), D=int(rng.choice([16, 64, 128])), out_of_place=True)


def test_step_lmhead_ragged_out_of_place_matches_oracle(b, ref):
    """sirllm_step_lmhead_ragged_out_of_place: the scores from hidden states and the output embedding matrix, the kept slots of
    every accepted stream in the second buffer pair; idle, empty and flagged streams, rows of 256 bytes and of other lengths."""
    rng = np.random.default_rng(78)
    pol = b.Policy(4, 20, 8, 0.9)
    run_ragged(b, ref, rng, 6, pol, 500, torch.bfloat16, [0, 10, 24, 40, 90, 0], [5, 22, 8, 0, 17, 0], lmhead_d=64, out_of_place=True)
    run_ragged(b, ref, rng, 3, pol, 777, torch.bfloat16, [100, 31, 0], [1, 1, 64], kv_dt=torch.bfloat16, D=128, lmhead_d=96,
               out_of_place=True)
    run_ragged(b, ref, rng, 2, pol, 300, torch.float16, [100, 31], [1, 1], kv_dt=torch.int16, D=5, lmhead_d=32, out_of_place=True)
    run_ragged(b, ref, rng, 4, pol, 100, torch.bfloat16, [40, -3, 50, -40], [5, 60, 8, 90], cap=100, new_cap=90, lmhead_d=64,
               out_of_place=True)
    run_ragged(b, ref, rng, 1, pol, 64, torch.bfloat16, [200], [0], lmhead_d=32, out_of_place=True)
    run_ragged(b, ref, rng, 3, b.Policy(4, 3068, 1024, 0.85), 2000, torch.bfloat16, [7168, 100, 4000], [1024, 1000, 96],
               L=2, H=4, D=128, kv_dt=torch.bfloat16, lmhead_d=128, out_of_place=True)


@pytest.mark.parametrize("tight_new", [True, False])
@pytest.mark.parametrize("held,new,pol_t", [
    # bound on n_cand in 8193..16384: sixteen slots per thread (select_ragged_kernel<1024, 16>)
    ([11000, 9000, 300, 12000, 8150], [1000, 700, 1000, 0, 43], (4, 6000, 1000, 0.9)),
    ([11800, 2000, 11000], [200, 64, 1000], (4, 4092, 0, 0.8)),                  # no recent window
    # bound in 16385..32768: thirty-two slots per thread (select_ragged_kernel<1024, 32>)
    ([30000, 500, 20000, 32000], [2000, 2000, 100, 768], (4, 16000, 2048, 0.9)),
    ([32768 - 54, 17000], [54, 54], (4, 1020, 0, 0.7)),                          # the documented limit of the call
])
def test_step_ragged_large_caches(b, ref, held, new, pol_t, tight_new):
    """Ragged steps whose largest stream holds 8193..32768 slots: the selecting workgroup then keeps 16 or 32
    slots per thread.  Streams of very different fill share the batch; tight and loose bounds on the new tokens."""
    rng = np.random.default_rng(len(held) * 1000 + held[0])
    run_ragged(b, ref, rng, len(held), b.Policy(*pol_t), 300, torch.bfloat16, held, new, L=1, H=2, D=64,
               kv_dt=torch.bfloat16, tight_new=tight_new)


@pytest.mark.parametrize("held,new,pol_t,kw", [
    # one slot past what one workgroup selects; a stream within its budget and an empty one in the same batch
    ([32768 - 53, 100, 0], [54, 54, 0], (4, 1020, 0, 0.7), {}),
    # streams above and below 32768 slots, one within the budget (only decayed), ragged last tiles
    ([39000, 20000, 33000, 8191], [800, 100, 1000, 1], (4, 30000, 1000, 0.9), {}),
    # no top-k part, and a top-k part that takes all but one middle slot
    ([50000, 100], [77, 5], (4, 0, 128, 0.9), {}),
    ([40000, 35000], [50, 1], (4, 40000, 45, 0.8), {}),
    # streams beyond the promised bounds (slots, new tokens, negative fill) are flagged and left alone
    ([39000, 60000, 36000, -5, 34000], [800, 10, 3000, 10, 100], (4, 30000, 1000, 0.9), {"cap": 41000, "new_cap": 1000}),
    # a 128K-slot budget with a ragged tail
    ([131072, 131000], [2048, 100], (4, 129020, 2048, 0.9), {}),
])
def test_step_ragged_above_one_workgroup(b, ref, held, new, pol_t, kw):
    """Ragged steps whose bound on the slots per stream exceeds 32768: every stream is then selected by the
    multi-workgroup kernels on its own sizes (Alg. 1 per stream), whatever it holds itself."""
    rng = np.random.default_rng(len(held) * 977 + abs(held[0]))
    run_ragged(b, ref, rng, len(held), b.Policy(*pol_t), 300, torch.bfloat16, held, new, L=1, H=2, D=16,
               kv_dt=torch.bfloat16, **kw)


@pytest.mark.parametrize("dt", [torch.bfloat16, torch.float16])
def test_step_lmhead_ragged_matches_oracle(b, ref, dt):
    """The ragged step fed with hidden states and the output embedding matrix (Sec. 3.2; Alg. 1 per stream): scores
    against the oracle's double-precision product, everything behind them bit exact given the scores."""
    rng = np.random.default_rng(4242)
    pol = b.Policy(4, 20, 8, 0.9)                       # budget 32
    # streams under, at and over the budget, empty streams, streams without new tokens; 1 to 3 token tiles
    run_ragged(b, ref, rng, 6, pol, 500, dt, [0, 10, 24, 40, 90, 0], [5, 22, 8, 0, 17, 0], lmhead_d=64)
    run_ragged(b, ref, rng, 3, pol, 777, dt, [100, 31, 0], [1, 1, 64], kv_dt=torch.bfloat16, D=128, lmhead_d=72)
    run_ragged(b, ref, rng, 1, pol, 64, dt, [200], [0], lmhead_d=64)
    run_ragged(b, ref, rng, 4, b.Policy(4, 1020, 0, 0.8), 1000, dt, [1024, 1000, 500, 1024], [54, 54, 54, 1],
               L=1, H=2, D=64, kv_dt=torch.bfloat16, lmhead_d=256)
    run_ragged(b, ref, rng, 3, b.Policy(4, 3068, 1024, 0.85), 2000, dt, [7168, 100, 4000], [300, 257, 96],
               L=1, H=2, D=64, kv_dt=torch.bfloat16, lmhead_d=128)
    # flagged streams: too many slots, too many new tokens, a negative slot count
    run_ragged(b, ref, rng, 3, pol, 100, dt, [10, 60, 20], [5, 30, 5], cap=40, tight_new=False, lmhead_d=64)
    run_ragged(b, ref, rng, 4, pol, 100, dt, [40, -3, 50, -40], [5, 60, 8, 90], cap=100, new_cap=90, lmhead_d=64)
    # a bound above 32768 slots per stream: the multi-workgroup selection behind the LM-head scores
    run_ragged(b, ref, rng, 3, b.Policy(4, 30000, 1000, 0.9), 300, dt, [39000, 20000, 33000], [80, 100, 130],
               L=1, H=2, D=16, kv_dt=torch.bfloat16, lmhead_d=64)


# ------------------------------------------------------------- scoring from chunks of columns
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16])
@pytest.mark.parametrize("n_rows,V,cuts", [
    (33, 1000, [0, 1000]),                       # a single chunk is the whole row
    (33, 1000, [0, 1, 500, 999, 1000]),          # one-column chunks at both ends
    (7, 32000, [0, 4000, 8000, 12000, 16000, 20000, 24000, 28000, 32000]),   # eight vocabulary shards
    (5, 128256, [0, 16032, 50001, 128256]),      # unequal shards, odd boundaries
    (64, 777, [0, 100, 101, 102, 640, 777]),
])
def test_score_from_column_chunks_matches_oracle(b, ref, dtype, n_rows, V, cuts):
    g = torch.Generator(device=DEV).manual_seed(V + n_rows)
    z = (torch.randn((n_rows, V), generator=g, device=DEV) * 3.0)
    z[::2, V // 3] += 9.0
    z = z.to(dtype)
    tok = torch.randint(0, V, (n_rows,), generator=g, device=DEV, dtype=torch.int32)
    tok[0], tok[-1] = 0, V - 1
    n_parts = len(cuts) - 1
    parts = torch.full((n_parts, 3 * n_rows + 5), 7.0, device=DEV)
    for p in range(n_parts):                      # column slices of the full tensor: ld stays V
        b.sirllm_score_partial(z[:, cuts[p]:cuts[p + 1]], cuts[p], tok, parts[p])
    out = torch.zeros(n_rows, device=DEV)
    b.sirllm_score_merge(parts, n_rows, out)
    torch.cuda.synchronize()
    want = ref.score(to_np(z), to_np(tok))
    assert_scores_close(to_np(out), want)
    # the whole-row kernel and the chunked path agree with each other to rounding as well
    whole = gpu_score(b, z, tok)
    np.testing.assert_allclose(to_np(out), whole, rtol=3e-6, atol=1e-6)
    assert (to_np(parts)[:, 3 * n_rows:] == 7.0).all()


def test_score_chunks_special_cases(b, ref):
    V = 600
    z = torch.zeros((5, V), device=DEV)
    z[0, :300] = -np.inf                         # a whole chunk of -inf merges as the neutral element
    z[1, :] = -np.inf                            # every chunk empty: NaN
    z[2, 450] = np.inf                           # +inf in one chunk: NaN
    z[3, 10] = np.nan
    tok = torch.tensor([400, 5, 0, 0, V + 3], dtype=torch.int32, device=DEV)   # last: no chunk holds the token
    parts = torch.zeros((2, 15), device=DEV)
    b.sirllm_score_partial(z[:, :300], 0, tok, parts[0])
    b.sirllm_score_partial(z[:, 300:], 300, tok, parts[1])
    out = torch.zeros(5, device=DEV)
    b.sirllm_score_merge(parts, 5, out)
    torch.cuda.synchronize()
    got = to_np(out)
    want = ref.score(to_np(z), to_np(tok))
    assert_scores_close(got, want)
    assert abs(got[0] - np.log(300)) < 1e-5 and np.isnan(got[1:]).all()


# ------------------------------------------------- caches beyond one workgroup (> 32768 slots)
LARGE_CASES = [
    # n_streams, n_held, n_new, n_sink, k, n_recent, decay, levels
    (1, 32000, 769, 4, 16000, 512, 0.9, 0),          # just over the one-workgroup limit
    (2, 39000, 1000, 4, 20000, 512, 0.9, 50),        # heavy ties across tiles
    (1, 131072, 2048, 4, 100000, 2048, 0.85, 0),     # a 128K-context cache
    (3, 50000, 0, 4, 1, 0, 0.5, 3),                  # k = 1 among three score levels
    (1, 60000, 5000, 0, 0, 1000, 0.9, 0),            # k = 0: sliding window
    (1, 60000, 5000, 4, 60995, 0, 1.0, 7),           # all but one middle slot kept
    (2, 500000, 24000, 4, 262144, 2048, 0.9, 1000),  # half a million slots
    (1, 40000, 100, 4, 50000, 512, 0.9, 0),          # under budget: keep-all path
    (1, 16777216 - 4096, 4096, 4, 8000000, 4096, 0.9, 0),   # SIRLLM_MAX_CAND slots, the documented limit
]


@pytest.mark.parametrize("case", LARGE_CASES, ids=[str(c[:6]) for c in LARGE_CASES])
def test_large_decay_select_matches_oracle(b, ref, case):
    n_streams, n_held, n_new, n_sink, k, n_recent, decay, levels = case
    rng = np.random.default_rng(n_held + 3 * n_new)
    n_cand = n_held + n_new
    if levels:
        E = (rng.integers(0, levels, (n_streams, n_cand)) / 8.0).astype(np.float32)
    else:
        E = rng.gamma(2.0, 2.0, (n_streams, n_cand)).astype(np.float32)
    pol = b.Policy(n_sink, k, n_recent, decay)
    n_keep = min(n_cand, n_sink + k + n_recent)
    Ed = torch.from_numpy(E).to(DEV)
    idx = torch.full((n_streams, n_keep + 3), -7, dtype=torch.int32, device=DEV)
    out = torch.full((n_streams, n_keep + 3), -7.0, device=DEV)
    nbytes = b.sirllm_workspace_bytes(n_streams, n_cand, 0, 0)
    ws = torch.full((nbytes + 256,), 0x5A, dtype=torch.uint8, device=DEV)     # dirty on purpose: the call clears what it needs
    for rep in range(2):                                                       # a second call on the used scratch
        b.sirllm_decay_select(Ed, n_held, n_new, pol, idx, out, workspace=ws[:nbytes] if nbytes else None)
        torch.cuda.synchronize()
        ri, ro = ref.decay_select(E, n_held, n_new, ref.Policy(*pol))
        np.testing.assert_array_equal(to_np(idx)[:, :n_keep], ri)
        np.testing.assert_array_equal(to_np(out)[:, :n_keep].view(np.uint32), ro.view(np.uint32))
        assert (to_np(idx)[:, n_keep:] == -7).all()
    assert bool((ws[nbytes:] == 0x5A).all())


def test_large_select_special_values(b, ref):
    n = 70000
    special = np.array([0.0, -0.0, 1e-41, -1e-41, np.inf, -np.inf, 3.0, -3.0, 2.5, 2.5], dtype=np.float32)
    E = np.tile(special, n // len(special))[None, :].copy()
    E.view(np.uint32)[0, 9] = 0x7FC00000
    E.view(np.uint32)[0, 50017] = 0xFFC00000
    ws = torch.zeros(b.sirllm_workspace_bytes(1, n, 0, 0), dtype=torch.uint8, device=DEV)
    for k in (1, 6999, 7000, 7001, 35000, 69000):
        pol = b.Policy(2, k, 2, 0.5)
        n_keep = 4 + k
        idx = torch.zeros((1, n_keep), dtype=torch.int32, device=DEV)
        out = torch.zeros((1, n_keep), device=DEV)
        b.sirllm_decay_select(torch.from_numpy(E).to(DEV), 35000, 35000, pol, idx, out, workspace=ws)
        torch.cuda.synchronize()
        ri, ro = ref.decay_select(E, 35000, 35000, ref.Policy(*pol))
        np.testing.assert_array_equal(to_np(idx), ri)
        np.testing.assert_array_equal(to_np(out).view(np.uint32), ro.view(np.uint32))


def test_step_with_a_large_cache(b, ref):
    # the whole step over 40000 candidate slots (selection through the multi-workgroup path), small planes
    import dataclasses
    w2 = dataclasses.replace(synth.WORKLOADS["tiny"], vocab=500)
    pol = b.Policy(4, 30000, 512, 0.9)
    S, n_held, n_new = 1, 39000, 1000
    g0 = torch.Generator(device=DEV).manual_seed(21)
    z = torch.randn((S * n_new, 500), generator=g0, device=DEV) * 2
    tok = torch.randint(0, 500, (S * n_new,), generator=g0, device=DEV, dtype=torch.int32)
    held = torch.rand((S, n_held), generator=g0, device=DEV) * 6
    k_c = torch.randn((S, 1, 2, n_held + n_new, 8), generator=g0, device=DEV)
    v_c = torch.randn((S, 1, 2, n_held + n_new, 8), generator=g0, device=DEV)
    n_cand, n_keep = n_held + n_new, 30516
    E = torch.full((S, n_cand), -5.0, device=DEV)
    E[:, :n_held] = held
    idx = torch.full((S, n_keep), -7, dtype=torch.int32, device=DEV)
    out = torch.full((S, n_keep), -7.0, device=DEV)
    k_d = torch.zeros((S, 1, 2, n_keep, 8), device=DEV)
    v_d = torch.zeros((S, 1, 2, n_keep, 8), device=DEV)
    ws = torch.zeros(b.sirllm_workspace_bytes(S, n_cand, S * n_new, 500), dtype=torch.uint8, device=DEV)
    with pytest.raises(b.SirllmError):                       # the scratch is not optional here
        b.sirllm_step(z, tok, 500, E, n_held, n_new, pol, k_c, v_c, k_d, v_d, idx, out)
    b.sirllm_step(z, tok, 500, E, n_held, n_new, pol, k_c, v_c, k_d, v_d, idx, out, workspace=ws)
    torch.cuda.synchronize()
    g = dict(E=E, idx=idx, out=out, k=k_d, v=v_d, n_keep=n_keep, evicted=True)
    check_step_against_oracle(b, ref, w2, z, tok, held, k_c, v_c, g, pol=pol)
