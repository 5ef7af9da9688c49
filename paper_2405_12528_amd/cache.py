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

    def reset(self):
        """Start a new dialogue: forget every slot (buffers are reused as they are)."""
        self.n_held = 0
