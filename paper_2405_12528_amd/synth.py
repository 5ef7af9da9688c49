"""Seeded synthetic inputs for the retention step: workload shapes and random tensors only.

This module holds none of the method's arithmetic.  It serves the GPU tests, the CPU tests
of the oracle and the benchmark alike, so both sides of a parity check see the same bytes.
The five workloads stand in for the dialogue workloads of the paper's experiments
(Sec. 4.2: cache of 512 or 1024 slots, 4 sink tokens, decay 0.5 to 1.0), scaled to the
shapes of 7B/8B-class decoders; the paper's datasets and model weights are not used.

Everything is drawn from a ``torch.Generator`` seeded by (seed, workload, turn, tensor kind),
on the device asked for.  CPU and GPU generators give different streams; parity tests always
copy the very bytes the GPU saw back to the host.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    vocab: int
    n_new: int                 # tokens per stream per turn
    logits_dtype: str          # "f32" | "bf16"
    sigma: float               # std-dev of the Gaussian part of the logits
    zipf_a: float              # >0: add -a*ln(rank) with a seeded rank permutation shared by all rows
    spike: float               # >0: add this to one random column ...
    spike_frac: float          # ... in this fraction of the rows
    n_sink: int
    n_topk: int
    n_recent: int
    decay: float
    n_layers: int
    n_kv_heads: int
    head_dim: int
    kv_dtype: str              # "f32" | "bf16"
    n_cand: int                # candidate slots per stream before compaction (steady state)
    n_streams: int = 1
    n_turns: int = 1
    checked_turns: tuple = field(default_factory=tuple)
    seed: int = 0
    d_model: int = 4096        # width of the final hidden state (LM-head scoring only)

    @property
    def budget(self) -> int:
        return self.n_sink + self.n_topk + self.n_recent

    @property
    def n_held(self) -> int:
        return self.n_cand - self.n_new

    @property
    def n_keep(self) -> int:
        return min(self.n_cand, self.budget)

    @property
    def logit_bytes(self) -> int:
        return 4 if self.logits_dtype == "f32" else 2

    @property
    def kv_elem_bytes(self) -> int:
        return 4 if self.kv_dtype == "f32" else 2

    def algorithmic_bytes(self) -> dict:
        """Bytes one step must move: each logit read once, one 4-byte score per new token, the held scores
        read once, index and score of every kept slot written once, each kept K/V row read once and written
        once (nothing for the rows that are dropped).  The 4-byte token ids are not counted."""
        rows = self.n_streams * self.n_new
        score = rows * self.vocab * self.logit_bytes + 4 * rows
        select = self.n_streams * (4 * self.n_held + 8 * self.n_keep)
        per_slot = self.n_layers * 2 * self.n_kv_heads * self.head_dim * self.kv_elem_bytes
        compact = 2 * self.n_streams * self.n_keep * per_slot if self.n_cand > self.budget else 0
        return dict(score=score, select=select, compact=compact, total=score + select + compact)


WORKLOADS = {
    # Tiny: 64 new tokens per turn over 4 turns, budget 32 = 4 + 20 + 8.
    "tiny": Workload("tiny", vocab=1000, n_new=64, logits_dtype="f32", sigma=2.0, zipf_a=0.0, spike=8.0,
                     spike_frac=0.3, n_sink=4, n_topk=20, n_recent=8, decay=0.9, n_layers=2, n_kv_heads=2,
                     head_dim=16, kv_dtype="f32", n_cand=96, n_turns=4, checked_turns=(1, 2, 3, 4), d_model=64),
    # Llama-2-7B-shaped: 32 layers x 32 heads x 128, V = 32000.
    "llama2_7b": Workload("llama2_7b", vocab=32000, n_new=512, logits_dtype="bf16", sigma=3.0, zipf_a=1.1,
                          spike=0.0, spike_frac=0.0, n_sink=4, n_topk=1532, n_recent=512, decay=0.9,
                          n_layers=32, n_kv_heads=32, head_dim=128, kv_dtype="bf16", n_cand=4096),
    # Mistral-7B-shaped (grouped-query attention: 8 KV heads).
    "mistral_7b": Workload("mistral_7b", vocab=32000, n_new=1024, logits_dtype="bf16", sigma=3.0, zipf_a=1.1,
                           spike=0.0, spike_frac=0.0, n_sink=4, n_topk=3068, n_recent=1024, decay=0.85,
                           n_layers=32, n_kv_heads=8, head_dim=128, kv_dtype="bf16", n_cand=8192),
    # Llama-3-8B-shaped: V = 128256, fp32 logits.  The benchmark's headline workload.
    "llama3_8b": Workload("llama3_8b", vocab=128256, n_new=2048, logits_dtype="f32", sigma=4.0, zipf_a=1.05,
                          spike=0.0, spike_frac=0.0, n_sink=4, n_topk=2044, n_recent=2048, decay=0.9,
                          n_layers=32, n_kv_heads=8, head_dim=128, kv_dtype="bf16", n_cand=8192),
    # Batched long dialogue: 32 streams x 200 turns of 256 tokens.
    "batched_dialogue": Workload("batched_dialogue", vocab=32000, n_new=256, logits_dtype="bf16", sigma=3.0,
                                 zipf_a=1.1, spike=0.0, spike_frac=0.0, n_sink=4, n_topk=1788, n_recent=256,
                                 decay=0.9, n_layers=32, n_kv_heads=32, head_dim=128, kv_dtype="bf16",
                                 n_cand=2304, n_streams=32, n_turns=200, checked_turns=(1, 50, 200)),
    # The paper's own operating point (Sec. 4.2, Rock-Paper-Scissors: ~54 tokens per round, cache
    # 1024 = 4 sink + 1020 entropy + 0 recent, decay 0.7-0.9, cache never reset), on a 7B-shaped K/V.
    # With no recent window every new token competes in Top_k: scoring, selection and gather form a
    # true dependency chain.
    "rps_dialogue": Workload("rps_dialogue", vocab=32000, n_new=54, logits_dtype="bf16", sigma=3.0, zipf_a=1.1,
                             spike=0.0, spike_frac=0.0, n_sink=4, n_topk=1020, n_recent=0, decay=0.8,
                             n_layers=32, n_kv_heads=32, head_dim=128, kv_dtype="bf16", n_cand=1078,
                             n_turns=2000, checked_turns=(1, 19, 20, 100, 300, 1000, 2000)),
    # A long-context cache: the Llama-3-8B shape with a 128K-slot budget (the pre-training length of its
    # long-context variants), 2048 new tokens per turn.  35 GB of K/V in flight per step; the selection runs
    # over 133120 candidate slots, beyond what one workgroup holds.
    # The Llama-3-8B shape with twice the budget: 10240 candidate slots, ten per lane of the selecting workgroup.
    "llama3_8k_budget": Workload("llama3_8k_budget", vocab=128256, n_new=2048, logits_dtype="f32", sigma=4.0, zipf_a=1.05,
                                 spike=0.0, spike_frac=0.0, n_sink=4, n_topk=6140, n_recent=2048, decay=0.9,
                                 n_layers=32, n_kv_heads=8, head_dim=128, kv_dtype="bf16", n_cand=10240),
    "llama3_128k": Workload("llama3_128k", vocab=128256, n_new=2048, logits_dtype="f32", sigma=4.0, zipf_a=1.05,
                            spike=0.0, spike_frac=0.0, n_sink=4, n_topk=129020, n_recent=2048, decay=0.9,
                            n_layers=32, n_kv_heads=8, head_dim=128, kv_dtype="bf16", n_cand=133120),
}

_KIND = {"logits": 1, "tokens": 2, "held": 3, "kv_k": 4, "kv_v": 5, "rank": 6, "spike": 7, "hidden": 8, "weight": 9}


def _torch_dtype(name: str):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def generator(w: Workload, kind: str, turn: int = 0, device="cpu") -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(((w.seed * 1000003 + turn) * 16 + _KIND[kind]) & 0x7FFFFFFFFFFFFFFF)
    return g


def make_logits(w: Workload, turn: int = 0, device="cpu", n_rows: int | None = None, ld: int | None = None):
    """[n_rows, ld] logits (columns >= vocab, if any, are filled with a sentinel that must be ignored)."""
    n_rows = w.n_streams * w.n_new if n_rows is None else n_rows
    ld = w.vocab if ld is None else ld
    g = generator(w, "logits", turn, device)
    out = torch.empty((n_rows, ld), dtype=_torch_dtype(w.logits_dtype), device=device)
    bias = None
    if w.zipf_a > 0:
        gr = generator(w, "rank", 0, "cpu")
        rank = torch.randperm(w.vocab, generator=gr).to(torch.float32) + 1.0
        bias = (-w.zipf_a * torch.log(rank)).to(device)
    chunk = max(1, (1 << 26) // max(ld, 1))          # ~256 MB of fp32 at a time
    gs = generator(w, "spike", turn, device)
    for r0 in range(0, n_rows, chunk):
        r1 = min(n_rows, r0 + chunk)
        z = torch.randn((r1 - r0, ld), generator=g, device=device, dtype=torch.float32) * w.sigma
        if bias is not None:
            z[:, :w.vocab] += bias
        if w.spike > 0:
            hit = torch.rand(r1 - r0, generator=gs, device=device) < w.spike_frac
            col = torch.randint(0, w.vocab, (r1 - r0,), generator=gs, device=device)
            rows = torch.nonzero(hit).flatten()
            z[rows, col[rows]] += w.spike
        if ld > w.vocab:
            z[:, w.vocab:] = 1.0e4                    # padding: a kernel that reads it is caught at once
        out[r0:r1] = z.to(out.dtype)
    return out


def make_lmhead(w: Workload, turn: int = 0, device="cpu", n_rows: int | None = None, dtype=torch.bfloat16,
                d_model: int | None = None, vocab: int | None = None):
    """Final hidden states [n_rows, d_model] and an output-embedding matrix [vocab, d_model] whose product
    has the same shape of distribution as make_logits: hidden = N(0, 1) + 1 in every coordinate, weight row
    v = N(0, sigma^2 / d_model) + bias_v / d_model with the workload's Zipf bias, so that
    hidden @ weight.T ~ bias_v + N(0, ~2 sigma^2).  The weights depend on the workload only, not on the turn."""
    n_rows = w.n_streams * w.n_new if n_rows is None else n_rows
    d_model = w.d_model if d_model is None else d_model
    vocab = w.vocab if vocab is None else vocab
    gh = generator(w, "hidden", turn, device)
    hidden = (torch.randn((n_rows, d_model), generator=gh, device=device, dtype=torch.float32) + 1.0).to(dtype)
    gw = generator(w, "weight", 0, device)
    weight = torch.empty((vocab, d_model), dtype=dtype, device=device)
    bias = None
    if w.zipf_a > 0:
        gr = generator(w, "rank", 0, "cpu")
        rank = torch.randperm(vocab, generator=gr).to(torch.float32) + 1.0
        bias = (-w.zipf_a * torch.log(rank) / d_model).to(device)
    chunk = max(1, (1 << 26) // d_model)
    for v0 in range(0, vocab, chunk):
        v1 = min(vocab, v0 + chunk)
        x = torch.randn((v1 - v0, d_model), generator=gw, device=device, dtype=torch.float32) * (w.sigma / math.sqrt(d_model))
        if bias is not None:
            x += bias[v0:v1, None]
        weight[v0:v1] = x.to(dtype)
    return hidden, weight


def make_token_ids(w: Workload, turn: int = 0, device="cpu", n_rows: int | None = None):
    n_rows = w.n_streams * w.n_new if n_rows is None else n_rows
    g = generator(w, "tokens", turn, device)
    return torch.randint(0, w.vocab, (n_rows,), generator=g, device=device, dtype=torch.int32)


def make_held_scores(w: Workload, n_held: int | None = None, device="cpu"):
    """[n_streams, n_held] positive, right-skewed scores that shrink with age: Gamma(2, scale 2)
    times decay**age, age = ceil((n_held - i) / n_new) turns ago."""
    n_held = w.n_held if n_held is None else n_held
    g = generator(w, "held", 0, "cpu")
    u = torch.rand((2, w.n_streams, n_held), generator=g, dtype=torch.float64).clamp_min(1e-300)
    gamma = -2.0 * (torch.log(u[0]) + torch.log(u[1]))          # sum of two Exp(scale 2)
    i = torch.arange(n_held, dtype=torch.float64)
    age = torch.ceil((n_held - i) / max(w.n_new, 1))
    return (gamma * torch.pow(torch.tensor(w.decay, dtype=torch.float64), age)).to(torch.float32).to(device)


def make_kv(w: Workload, n_pos: int | None = None, turn: int = 0, device="cpu", which: str = "k"):
    """[n_streams, n_layers, n_kv_heads, n_pos, head_dim] ~ N(0, 1) in the workload's K/V dtype."""
    n_pos = w.n_cand if n_pos is None else n_pos
    g = generator(w, "kv_" + which, turn, device)
    shape = (w.n_streams, w.n_layers, w.n_kv_heads, n_pos, w.head_dim)
    out = torch.empty(shape, dtype=_torch_dtype(w.kv_dtype), device=device)
    flat = out.view(-1)
    chunk = 1 << 28
    for o in range(0, flat.numel(), chunk):
        n = min(chunk, flat.numel() - o)
        flat[o:o + n] = torch.randn(n, generator=g, device=device, dtype=torch.float32).to(out.dtype)
    return out


def tagged_kv(n_streams: int, n_layers: int, n_kv_heads: int, n_pos: int, head_dim: int, which: int,
              dtype=torch.int32, device="cpu"):
    """A K/V payload whose every element names its own coordinates, so a misrouted row
    identifies itself: value = ((((which*S + s)*L + l)*H + h)*P + p)*D + d  (mod 2**31)."""
    s = torch.arange(n_streams, dtype=torch.int64).view(-1, 1, 1, 1, 1)
    l = torch.arange(n_layers, dtype=torch.int64).view(1, -1, 1, 1, 1)
    h = torch.arange(n_kv_heads, dtype=torch.int64).view(1, 1, -1, 1, 1)
    p = torch.arange(n_pos, dtype=torch.int64).view(1, 1, 1, -1, 1)
    d = torch.arange(head_dim, dtype=torch.int64).view(1, 1, 1, 1, -1)
    v = ((((which * n_streams + s) * n_layers + l) * n_kv_heads + h) * n_pos + p) * head_dim + d
    return (v % (1 << 31)).to(dtype).to(device)


def describe(w: Workload) -> str:
    b = w.algorithmic_bytes()
    return (f"{w.name}: V={w.vocab} {w.logits_dtype} logits, {w.n_streams} stream(s) x {w.n_new} new tokens, "
            f"budget {w.budget} = {w.n_sink}+{w.n_topk}+{w.n_recent}, decay {w.decay}, "
            f"KV {w.n_layers}x{w.n_kv_heads}x{w.head_dim} {w.kv_dtype}, {w.n_cand} candidates, "
            f"{b['total'] / 1e9:.4f} GB/step")


__all__ = ["Workload", "WORKLOADS", "generator", "make_logits", "make_token_ids", "make_held_scores",
           "make_kv", "make_lmhead", "tagged_kv", "describe", "math"]
