"""Device-side state of a batch of dialogue streams across turns: ping-pong K/V buffers, the
entropy cache and the slot count, with one method that runs a whole retention step.

Plumbing only: every number is produced by the library's kernels (``binding.sirllm_step``).
The two K/V buffer pairs are allocated once, sized for budget + max_new slots; compaction is
out of place, so a step that evicts writes the other pair and the roles swap (paper Sec. 3.3,
Algorithm 1: the cache after an eviction holds exactly the budget).
"""
from __future__ import annotations

import torch

from . import binding as b


class RetentiveCache:
    def __init__(self, n_streams: int, n_layers: int, n_kv_heads: int, head_dim: int, policy, max_new: int,
                 kv_dtype=torch.bfloat16, device="cuda:0"):
        self.policy = b.Policy(*policy)
        self.budget = self.policy.n_sink + self.policy.n_topk + self.policy.n_recent
        self.capacity = self.budget + max_new
        if self.capacity > b.SIRLLM_MAX_CAND:
            raise ValueError(f"budget + max_new = {self.capacity} exceeds SIRLLM_MAX_CAND = {b.SIRLLM_MAX_CAND}")
        self.n_streams, self.max_new, self.device = n_streams, max_new, device
        shape = (n_streams, n_layers, n_kv_heads, self.capacity, head_dim)
        self._k = [torch.zeros(shape, dtype=kv_dtype, device=device) for _ in range(2)]
        self._v = [torch.zeros(shape, dtype=kv_dtype, device=device) for _ in range(2)]
        self._scores = [torch.zeros((n_streams, self.capacity), device=device) for _ in range(2)]
        self.kept_idx = torch.zeros((n_streams, self.capacity), dtype=torch.int32, device=device)
        self._cur = 0
        self.n_held = 0
        nbytes = b.sirllm_workspace_bytes(n_streams, self.capacity, n_streams * max_new, 1 << 20)
        self._ws = torch.zeros(nbytes, dtype=torch.uint8, device=device) if nbytes else None
        self._lm_ws = None                             # scratch of step_from_hidden, sized on first use

    # -- views of the live state ------------------------------------------------------------
    @property
    def k(self) -> torch.Tensor:
        """[streams, layers, kv_heads, capacity, head_dim]; slots [0, n_held) are live."""
        return self._k[self._cur]

    @property
    def v(self) -> torch.Tensor:
        return self._v[self._cur]

    @property
    def scores(self) -> torch.Tensor:
        """[streams, capacity]; entries [0, n_held) are the (decayed) token entropies of the live slots."""
        return self._scores[self._cur]

    def new_kv_slots(self, n_new: int):
        """The K and V views the model writes this turn's n_new tokens into, before step()."""
        if n_new > self.max_new or self.n_held + n_new > self.capacity:
            raise ValueError("more new tokens than the cache was sized for")
        s = slice(self.n_held, self.n_held + n_new)
        return self.k[:, :, :, s, :], self.v[:, :, :, s, :]

    # -- one turn ---------------------------------------------------------------------------
    def step(self, logits: torch.Tensor, token_ids: torch.Tensor, vocab: int, stream=None) -> bool:
        """Score the n_new = logits.shape[0] / n_streams tokens whose K/V sit at slots
        [n_held, n_held + n_new), decay, select and compact.  Returns True when slots were evicted
        (kept_idx[:, :budget] then lists the kept slots of the pre-step cache)."""
        n_new = logits.shape[0] // self.n_streams
        if n_new * self.n_streams != logits.shape[0] or n_new > self.max_new:
            raise ValueError("logits must hold n_streams * n_new rows with n_new <= max_new")
        cur, oth = self._cur, 1 - self._cur
        n_cand = self.n_held + n_new
        n_keep = b.sirllm_step(logits, token_ids, vocab, self._scores[cur], self.n_held, n_new, self.policy,
                               self._k[cur], self._v[cur], self._k[oth], self._v[oth], self.kept_idx,
                               self._scores[oth], workspace=self._ws, stream=stream)
        evicted = n_cand > n_keep
        # scores always move to the other array (decayed); K/V only when something was evicted
        if evicted:
            self._cur = oth
        else:
            self._scores[cur], self._scores[oth] = self._scores[oth], self._scores[cur]
        self.n_held = n_keep
        return evicted

    def step_from_hidden(self, hidden: torch.Tensor, weight: torch.Tensor, token_ids: torch.Tensor, stream=None) -> bool:
        """step() with the scores taken straight from the final hidden states [n_streams * n_new, d_model] and the
        output embedding matrix [vocab, d_model] (bf16 or f16): the logits are never stored."""
        n_new = hidden.shape[0] // self.n_streams
        if n_new * self.n_streams != hidden.shape[0] or n_new > self.max_new:
            raise ValueError("hidden must hold n_streams * n_new rows with n_new <= max_new")
        cur, oth = self._cur, 1 - self._cur
        n_cand = self.n_held + n_new
        need = b.sirllm_step_lmhead_workspace_bytes(self.n_streams, n_cand, hidden.shape[0], weight.shape[0])
        if self._lm_ws is None or self._lm_ws.numel() < need:
            self._lm_ws = torch.empty(max(need, 256), dtype=torch.uint8, device=self.device)
        n_keep = b.sirllm_step_lmhead(hidden, weight, token_ids, self._scores[cur], self.n_held, n_new, self.policy,
                                      self._k[cur], self._v[cur], self._k[oth], self._v[oth], self.kept_idx,
                                      self._scores[oth], self._lm_ws, stream=stream)
        evicted = n_cand > n_keep
        if evicted:
            self._cur = oth
        else:
            self._scores[cur], self._scores[oth] = self._scores[oth], self._scores[cur]
        self.n_held = n_keep
        return evicted

    def reset(self):
        """Start a new dialogue: forget every slot (buffers are reused as they are)."""
        self.n_held = 0


class LayeredRetentiveCache:
    """The same state with K and V held as one [streams, kv_heads, capacity, head_dim] tensor PER LAYER, the way model
    code usually keeps its past keys and values; compacted in place.  A step is sirllm_score_select followed by
    sirllm_compact_kv_inplace_layers."""

    def __init__(self, n_streams: int, n_layers: int, n_kv_heads: int, head_dim: int, policy, max_new: int,
                 kv_dtype=torch.bfloat16, device="cuda:0"):
        self.policy = b.Policy(*policy)
        self.budget = self.policy.n_sink + self.policy.n_topk + self.policy.n_recent
        self.capacity = self.budget + max_new
        self.n_streams, self.max_new, self.device = n_streams, max_new, device
        shape = (n_streams, n_kv_heads, self.capacity, head_dim)
        self.k = [torch.zeros(shape, dtype=kv_dtype, device=device) for _ in range(n_layers)]
        self.v = [torch.zeros(shape, dtype=kv_dtype, device=device) for _ in range(n_layers)]
        self._scores = [torch.zeros((n_streams, self.capacity), device=device) for _ in range(2)]
        self.kept_idx = torch.zeros((n_streams, self.capacity), dtype=torch.int32, device=device)
        self._cur = 0
        self.n_held = 0
        nbytes = max(b.sirllm_workspace_bytes(n_streams, self.capacity, n_streams * max_new, 1 << 20),
                     b.SIRLLM_INPLACE_WORKSPACE_BYTES)
        self._ws = torch.zeros(nbytes, dtype=torch.uint8, device=device)

    @property
    def scores(self) -> torch.Tensor:
        """[streams, capacity]; entries [0, n_held) are the (decayed) token entropies of the live slots."""
        return self._scores[self._cur]

    def new_kv_slots(self, layer: int, n_new: int):
        """The K and V views of one layer that the model writes this turn's n_new tokens into, before step()."""
        if n_new > self.max_new or self.n_held + n_new > self.capacity:
            raise ValueError("more new tokens than the cache was sized for")
        s = slice(self.n_held, self.n_held + n_new)
        return self.k[layer][:, :, s, :], self.v[layer][:, :, s, :]

    def step(self, logits: torch.Tensor, token_ids: torch.Tensor, vocab: int, stream=None) -> bool:
        """Score the n_new = logits.shape[0] / n_streams tokens at slots [n_held, n_held + n_new), decay, select and
        compact every layer in place.  Returns True when slots were evicted."""
        n_new = logits.shape[0] // self.n_streams
        if n_new * self.n_streams != logits.shape[0] or n_new > self.max_new:
            raise ValueError("logits must hold n_streams * n_new rows with n_new <= max_new")
        cur, oth = self._cur, 1 - self._cur
        n_cand = self.n_held + n_new
        n_keep = b.sirllm_score_select(logits, token_ids, vocab, self._scores[cur], self.n_held, n_new, self.policy,
                                       self.kept_idx, self._scores[oth], workspace=self._ws, stream=stream)
        evicted = n_cand > n_keep
        if evicted:
            b.sirllm_compact_kv_inplace_layers(self.k, self.v, self.kept_idx, n_keep, n_src=n_cand, workspace=self._ws,
                                               stream=stream)
        self._cur = oth
        self.n_held = n_keep
        return evicted

    def reset(self):
        """Start a new dialogue: forget every slot (buffers are reused as they are)."""
        self.n_held = 0


class RaggedRetentiveCache:
    """The same state for a serving batch whose streams are at different turns: every stream has its
    own slot count and takes its own number of new tokens per step; K/V are compacted in place, so
    there is one K/V buffer pair instead of two.  Slot counts are mirrored on the host (they are plain
    arithmetic: min(n_held + n_new, budget)) so that no step needs a device read-back."""

    def __init__(self, n_streams: int, n_layers: int, n_kv_heads: int, head_dim: int, policy, max_new: int,
                 kv_dtype=torch.bfloat16, device="cuda:0"):
        self.policy = b.Policy(*policy)
        self.budget = self.policy.n_sink + self.policy.n_topk + self.policy.n_recent
        self.capacity = self.budget + max_new
        self.n_streams, self.max_new, self.device = n_streams, max_new, device
        shape = (n_streams, n_layers, n_kv_heads, self.capacity, head_dim)
        self.k = torch.zeros(shape, dtype=kv_dtype, device=device)
        self.v = torch.zeros(shape, dtype=kv_dtype, device=device)
        self._scores = [torch.zeros((n_streams, self.capacity), device=device) for _ in range(2)]
        self._held_dev = [torch.zeros(n_streams, dtype=torch.int32, device=device) for _ in range(2)]
        self.kept_idx = torch.zeros((n_streams, self.capacity), dtype=torch.int32, device=device)
        self._cur = 0
        self.n_held = [0] * n_streams                  # host mirror
        # the multi-workgroup selection's scratch (above 32768 slots per stream) and the in-place compaction's
        # ticket counter live in the workspace
        nbytes = max(b.sirllm_workspace_bytes(n_streams, self.capacity, n_streams * max_new, 1 << 20),
                     b.SIRLLM_INPLACE_WORKSPACE_BYTES)
        self._ws = torch.zeros(nbytes, dtype=torch.uint8, device=device) if nbytes else None
        self._lm_ws = None                             # sized on the first step_from_hidden

    @property
    def scores(self) -> torch.Tensor:
        """[streams, capacity]; entries [0, n_held[s]) of row s are live."""
        return self._scores[self._cur]

    def new_kv_slots(self, s: int, n_new: int):
        """K and V views for the n_new tokens stream s appends this step."""
        if n_new > self.max_new:
            raise ValueError("more new tokens than the cache was sized for")
        sl = slice(self.n_held[s], self.n_held[s] + n_new)
        return self.k[s, :, :, sl, :], self.v[s, :, :, sl, :]

    def step(self, logits: torch.Tensor, token_ids: torch.Tensor, vocab: int, n_new, stream=None):
        """n_new[s] tokens per stream (0 for idle streams); logits rows are concatenated stream by stream."""
        if len(n_new) != self.n_streams or max(n_new) > self.max_new or min(n_new) < 0:
            raise ValueError("n_new must give 0..max_new tokens for every stream")
        cu = [0]
        for n in n_new:
            cu.append(cu[-1] + int(n))
        cu_dev = torch.tensor(cu, dtype=torch.int32, device=self.device)
        max_cand = max(h + int(n) for h, n in zip(self.n_held, n_new))
        cur, oth = self._cur, 1 - self._cur
        b.sirllm_step_ragged(logits, token_ids, vocab, self._scores[cur], self._held_dev[cur], cu_dev, cu[-1],
                             max_cand, self.policy, self.k, self.v, self.kept_idx, self._scores[oth],
                             self._held_dev[oth], max_new=max(int(n) for n in n_new), workspace=self._ws,
                             stream=stream)
        self._cur = oth
        evicted = [h + int(n) > self.budget for h, n in zip(self.n_held, n_new)]
        self.n_held = [min(h + int(n), self.budget) for h, n in zip(self.n_held, n_new)]
        return evicted

    def step_from_hidden(self, hidden: torch.Tensor, weight: torch.Tensor, token_ids: torch.Tensor, n_new, stream=None):
        """step() with the scores taken straight from the final hidden states [sum(n_new), d_model] (rows concatenated
        stream by stream) and the output embedding matrix [vocab, d_model] (bf16 or f16): no logits are stored."""
        if len(n_new) != self.n_streams or max(n_new) > self.max_new or min(n_new) < 0:
            raise ValueError("n_new must give 0..max_new tokens for every stream")
        cu = [0]
        for n in n_new:
            cu.append(cu[-1] + int(n))
        cu_dev = torch.tensor(cu, dtype=torch.int32, device=self.device)
        max_cand = max(h + int(n) for h, n in zip(self.n_held, n_new))
        need = b.sirllm_step_lmhead_ragged_workspace_bytes(self.n_streams, max_cand, cu[-1], weight.shape[0])
        if self._lm_ws is None or self._lm_ws.numel() < need:
            self._lm_ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        cur, oth = self._cur, 1 - self._cur
        b.sirllm_step_lmhead_ragged(hidden, weight, token_ids, self._scores[cur], self._held_dev[cur], cu_dev, cu[-1],
                                    max_cand, self.policy, self.k, self.v, self.kept_idx, self._scores[oth],
                                    self._held_dev[oth], self._lm_ws, max_new=max(int(n) for n in n_new), stream=stream)
        self._cur = oth
        evicted = [h + int(n) > self.budget for h, n in zip(self.n_held, n_new)]
        self.n_held = [min(h + int(n), self.budget) for h, n in zip(self.n_held, n_new)]
        return evicted

    def reset(self, s: int):
        """Start a new dialogue in stream s."""
        self.n_held[s] = 0
        self._held_dev[self._cur][s] = 0


class RaggedTwoBufferCache:
    """RaggedRetentiveCache with the K/V movement out of place: two K/V buffer pairs that swap roles every step.  Every
    stream's kept slots are written to the other pair (compacted when over budget, as they are otherwise), so the whole
    batch always lives in one pair; costs twice the K/V memory and moves the cache 5 to 14 % faster than the in-place
    walk.  (A stream that is reset, or idle, simply has its slots copied along.)"""

    def __init__(self, n_streams: int, n_layers: int, n_kv_heads: int, head_dim: int, policy, max_new: int,
                 kv_dtype=torch.bfloat16, device="cuda:0"):
        self.policy = b.Policy(*policy)
        self.budget = self.policy.n_sink + self.policy.n_topk + self.policy.n_recent
        self.capacity = self.budget + max_new
        self.n_streams, self.max_new, self.device = n_streams, max_new, device
        shape = (n_streams, n_layers, n_kv_heads, self.capacity, head_dim)
        self._k = [torch.zeros(shape, dtype=kv_dtype, device=device) for _ in range(2)]
        self._v = [torch.zeros(shape, dtype=kv_dtype, device=device) for _ in range(2)]
        self._scores = [torch.zeros((n_streams, self.capacity), device=device) for _ in range(2)]
        self._held_dev = [torch.zeros(n_streams, dtype=torch.int32, device=device) for _ in range(2)]
        self.kept_idx = torch.zeros((n_streams, self.capacity), dtype=torch.int32, device=device)
        self._cur = 0
        self.n_held = [0] * n_streams                  # host mirror
        nbytes = b.sirllm_workspace_bytes(n_streams, self.capacity, n_streams * max_new, 1 << 20)
        self._ws = torch.zeros(nbytes, dtype=torch.uint8, device=device) if nbytes else None
        self._lm_ws = None

    @property
    def k(self) -> torch.Tensor:
        """[streams, layers, kv_heads, capacity, head_dim]; slots [0, n_held[s]) of stream s are live."""
        return self._k[self._cur]

    @property
    def v(self) -> torch.Tensor:
        return self._v[self._cur]

    @property
    def scores(self) -> torch.Tensor:
        """[streams, capacity]; entries [0, n_held[s]) of row s are live."""
        return self._scores[self._cur]

    def new_kv_slots(self, s: int, n_new: int):
        """K and V views for the n_new tokens stream s appends this step."""
        if n_new > self.max_new:
            raise ValueError("more new tokens than the cache was sized for")
        sl = slice(self.n_held[s], self.n_held[s] + n_new)
        return self.k[s, :, :, sl, :], self.v[s, :, :, sl, :]

    def step(self, logits: torch.Tensor, token_ids: torch.Tensor, vocab: int, n_new, stream=None):
        """n_new[s] tokens per stream (0 for idle streams); logits rows are concatenated stream by stream."""
        if len(n_new) != self.n_streams or max(n_new) > self.max_new or min(n_new) < 0:
            raise ValueError("n_new must give 0..max_new tokens for every stream")
        cu = [0]
        for n in n_new:
            cu.append(cu[-1] + int(n))
        cu_dev = torch.tensor(cu, dtype=torch.int32, device=self.device)
        max_cand = max(h + int(n) for h, n in zip(self.n_held, n_new))
        cur, oth = self._cur, 1 - self._cur
        b.sirllm_step_ragged_out_of_place(logits, token_ids, vocab, self._scores[cur], self._held_dev[cur], cu_dev, cu[-1],
                                          max_cand, self.policy, self._k[cur], self._v[cur], self._k[oth], self._v[oth],
                                          self.kept_idx, self._scores[oth], self._held_dev[oth],
                                          max_new=max(int(n) for n in n_new), workspace=self._ws, stream=stream)
        self._cur = oth
        evicted = [h + int(n) > self.budget for h, n in zip(self.n_held, n_new)]
        self.n_held = [min(h + int(n), self.budget) for h, n in zip(self.n_held, n_new)]
        return evicted

    def step_from_hidden(self, hidden: torch.Tensor, weight: torch.Tensor, token_ids: torch.Tensor, n_new, stream=None):
        """step() with the scores taken straight from the final hidden states [sum(n_new), d_model] (rows concatenated
        stream by stream) and the output embedding matrix [vocab, d_model] (bf16 or f16): no logits are stored."""
        if len(n_new) != self.n_streams or max(n_new) > self.max_new or min(n_new) < 0:
            raise ValueError("n_new must give 0..max_new tokens for every stream")
        cu = [0]
        for n in n_new:
            cu.append(cu[-1] + int(n))
        cu_dev = torch.tensor(cu, dtype=torch.int32, device=self.device)
        max_cand = max(h + int(n) for h, n in zip(self.n_held, n_new))
        need = b.sirllm_step_lmhead_ragged_workspace_bytes(self.n_streams, max_cand, cu[-1], weight.shape[0])
        if self._lm_ws is None or self._lm_ws.numel() < need:
            self._lm_ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        cur, oth = self._cur, 1 - self._cur
        b.sirllm_step_lmhead_ragged_out_of_place(hidden, weight, token_ids, self._scores[cur], self._held_dev[cur], cu_dev,
                                                 cu[-1], max_cand, self.policy, self._k[cur], self._v[cur], self._k[oth],
                                                 self._v[oth], self.kept_idx, self._scores[oth], self._held_dev[oth],
                                                 self._lm_ws, max_new=max(int(n) for n in n_new), stream=stream)
        self._cur = oth
        evicted = [h + int(n) > self.budget for h, n in zip(self.n_held, n_new)]
        self.n_held = [min(h + int(n), self.budget) for h, n in zip(self.n_held, n_new)]
        return evicted

    def reset(self, s: int):
        """Start a new dialogue in stream s."""
        self.n_held[s] = 0
        self._held_dev[self._cur][s] = 0
