"""numpy front end of the C oracle (oracle/sirllm_ref.c).  TEST INFRASTRUCTURE ONLY.

Arrays are numpy, host memory.  bfloat16 data is carried as ``uint16`` bit patterns.  The
functions only marshal arguments; every number comes out of the C code.
"""
from __future__ import annotations

import ctypes as C
import os
from collections import namedtuple

import numpy as np

from . import build as _build

Policy = namedtuple("Policy", "n_sink n_topk n_recent decay")

F32, BF16, F16 = 0, 1, 2


class _CPolicy(C.Structure):
    _fields_ = [("n_sink", C.c_int32), ("n_topk", C.c_int32), ("n_recent", C.c_int32), ("decay", C.c_float)]


class _CLayout(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("elem_bytes", C.c_int32), ("stride_stream", C.c_int64), ("stride_layer", C.c_int64),
                ("stride_head", C.c_int64), ("stride_pos", C.c_int64)]


_lib = None


def load(path):
    """Open a build of the oracle and declare its signatures."""
    L = C.CDLL(path)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    L.sirllm_ref_score.argtypes = [vp, C.c_int, i64, i32, i64, vp, vp]
    L.sirllm_ref_lmhead_score.argtypes = [vp, i64, vp, i64, C.c_int, i32, i64, i32, vp, vp]
    L.sirllm_ref_lmhead_score.restype = C.c_int
    L.sirllm_ref_decay_select.argtypes = [vp, i64, i32, i32, i32, C.POINTER(_CPolicy), vp, i64, vp, i64]
    L.sirllm_ref_compact_kv.argtypes = [vp, vp, C.POINTER(_CLayout), i32, vp, vp, C.POINTER(_CLayout),
                                        vp, i64, i32, i32]
    L.sirllm_ref_step.argtypes = [vp, C.c_int, i32, i64, vp, vp, i64, i32, i32, i32, C.POINTER(_CPolicy),
                                  vp, vp, C.POINTER(_CLayout), vp, vp, C.POINTER(_CLayout),
                                  vp, i64, vp, i64]
    L.sirllm_ref_compact_kv_inplace.argtypes = [vp, vp, C.POINTER(_CLayout), i32, vp, i64, i32, i32]
    L.sirllm_ref_compact_kv_inplace.restype = C.c_int
    L.sirllm_ref_baseline_select.argtypes = [C.c_int, i32, i32, C.POINTER(_CPolicy), C.c_uint64, C.c_uint64, vp, i64,
                                             C.POINTER(i32)]
    L.sirllm_ref_baseline_select.restype = C.c_int
    L.sirllm_ref_philox4x32_10.argtypes = [C.POINTER(C.c_uint32 * 4), C.POINTER(C.c_uint32 * 2),
                                           C.POINTER(C.c_uint32 * 4)]
    L.sirllm_ref_philox4x32_10.restype = None
    for f in (L.sirllm_ref_score, L.sirllm_ref_decay_select, L.sirllm_ref_compact_kv, L.sirllm_ref_step,
              L.sirllm_ref_set_threads, L.sirllm_ref_get_threads):
        f.restype = C.c_int
    L.sirllm_ref_set_threads.argtypes = [C.c_int]
    return L


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            path = _build.build()
        _lib = load(path)
    return _lib


def set_threads(n: int) -> int:
    return lib().sirllm_ref_set_threads(int(n))


def _ptr(a):
    return None if a is None else a.ctypes.data


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what}: invalid argument (rc={rc})")


def _logits_dtype(logits):
    if logits.dtype == np.float32:
        return F32
    if logits.dtype == np.uint16:
        return BF16
    if logits.dtype == np.float16:
        return F16
    raise TypeError("logits must be float32, float16 or uint16 (bfloat16 bit patterns)")


def _cpolicy(p):
    return _CPolicy(int(p.n_sink), int(p.n_topk), int(p.n_recent), float(p.decay))


def n_keep_of(n_cand: int, p) -> int:
    return min(int(n_cand), int(p.n_sink) + int(p.n_topk) + int(p.n_recent))


def score(logits: np.ndarray, token_ids: np.ndarray, vocab: int | None = None) -> np.ndarray:
    """Token entropy of each row's token; logits is [n_rows, ld] (ld >= vocab)."""
    assert logits.ndim == 2 and logits.flags.c_contiguous
    n_rows, ld = logits.shape
    vocab = ld if vocab is None else int(vocab)
    tok = np.ascontiguousarray(token_ids, dtype=np.int32)
    assert tok.shape == (n_rows,)
    out = np.empty(n_rows, dtype=np.float32)
    _check(lib().sirllm_ref_score(_ptr(logits), _logits_dtype(logits), n_rows, vocab, ld, _ptr(tok), _ptr(out)),
           "score")
    return out


def lmhead_score(hidden: np.ndarray, weight: np.ndarray, token_ids: np.ndarray, d_model: int | None = None,
                 vocab: int | None = None) -> np.ndarray:
    """Token entropy with the logits written as hidden @ weight.T: hidden is [n_rows, ld_h], weight is
    [vocab, ld_w] (row v = output embedding of token v), same element type (bf16 as uint16 bits)."""
    assert hidden.ndim == 2 and weight.ndim == 2 and hidden.flags.c_contiguous and weight.flags.c_contiguous
    assert hidden.dtype == weight.dtype
    n_rows, ld_h = hidden.shape
    d_model = min(ld_h, weight.shape[1]) if d_model is None else int(d_model)
    vocab = weight.shape[0] if vocab is None else int(vocab)
    assert vocab <= weight.shape[0]
    tok = np.ascontiguousarray(token_ids, dtype=np.int32)
    assert tok.shape == (n_rows,)
    out = np.empty(n_rows, dtype=np.float32)
    _check(lib().sirllm_ref_lmhead_score(_ptr(hidden), ld_h, _ptr(weight), weight.shape[1], _logits_dtype(hidden),
                                         d_model, n_rows, vocab, _ptr(tok), _ptr(out)), "lmhead_score")
    return out


def decay_select(scores: np.ndarray, n_held: int, n_new: int, policy):
    """scores is [n_streams, >= n_held+n_new] float32.  Returns (kept_idx, scores_out), each [n_streams, n_keep]."""
    scores = np.ascontiguousarray(scores, dtype=np.float32)
    assert scores.ndim == 2
    n_streams, stride = scores.shape
    n_cand = n_held + n_new
    assert stride >= n_cand
    n_keep = n_keep_of(n_cand, policy)
    kept = np.full((n_streams, max(n_keep, 1)), -1, dtype=np.int32)
    out = np.full((n_streams, max(n_keep, 1)), np.nan, dtype=np.float32)
    cp = _cpolicy(policy)
    _check(lib().sirllm_ref_decay_select(_ptr(scores), stride, n_streams, n_held, n_new, C.byref(cp),
                                         _ptr(kept), kept.shape[1], _ptr(out), out.shape[1]), "decay_select")
    return kept[:, :n_keep], out[:, :n_keep]


STREAM, INTERVAL, RANDOM = 0, 1, 2


def baseline_select(kind: int, n_streams: int, n_cand: int, policy, seed: int = 0, turn: int = 0) -> np.ndarray:
    """Kept slots [n_streams, n_keep] of a baseline policy (StreamLLM / IntervalLLM / RandomLLM)."""
    cp = _cpolicy(policy)
    cap = max(1, min(n_cand, int(policy.n_sink) + int(policy.n_topk) + int(policy.n_recent)))
    kept = np.full((max(n_streams, 1), cap), -1, dtype=np.int32)
    n_keep = C.c_int32(-1)
    _check(lib().sirllm_ref_baseline_select(int(kind), n_streams, n_cand, C.byref(cp), int(seed), int(turn),
                                            _ptr(kept), cap, C.byref(n_keep)), "baseline_select")
    return kept[:n_streams, :n_keep.value]


def philox4x32_10(ctr, key):
    c = (C.c_uint32 * 4)(*ctr)
    k = (C.c_uint32 * 2)(*key)
    out = (C.c_uint32 * 4)()
    lib().sirllm_ref_philox4x32_10(C.byref(c), C.byref(k), C.byref(out))
    return [int(x) for x in out]


def _layout_of(a: np.ndarray) -> _CLayout:
    """a is [streams, layers, heads, slots, head_dim] with the last axis contiguous."""
    assert a.ndim == 5
    es = a.dtype.itemsize
    st = [s // es for s in a.strides]
    assert st[4] == 1 or a.shape[4] <= 1
    return _CLayout(a.shape[1], a.shape[2], a.shape[4], es, st[0], st[1], st[2], st[3])


def compact_kv(k_src: np.ndarray, v_src: np.ndarray | None, kept_idx: np.ndarray, n_src: int | None = None):
    """Gather slots kept_idx[s, :] of [streams, layers, heads, slots, head_dim] caches."""
    kept_idx = np.ascontiguousarray(kept_idx, dtype=np.int32)
    n_streams, n_keep = kept_idx.shape
    assert k_src.shape[0] == n_streams
    n_src = k_src.shape[3] if n_src is None else int(n_src)
    shape = k_src.shape[:3] + (n_keep,) + k_src.shape[4:]
    k_dst = np.empty(shape, dtype=k_src.dtype)
    v_dst = None if v_src is None else np.empty(shape, dtype=v_src.dtype)
    ls, ld = _layout_of(k_src), _layout_of(k_dst)
    if v_src is not None:
        assert v_src.shape == k_src.shape and v_src.strides == k_src.strides and v_src.dtype == k_src.dtype
    _check(lib().sirllm_ref_compact_kv(_ptr(k_src), _ptr(v_src), C.byref(ls), n_src, _ptr(k_dst), _ptr(v_dst),
                                       C.byref(ld), _ptr(kept_idx), max(n_keep, 1) if n_keep else 1,
                                       n_streams, n_keep), "compact_kv")
    return k_dst, v_dst


def compact_kv_inplace(k: np.ndarray, v: np.ndarray | None, kept_idx: np.ndarray, n_src: int | None = None):
    """In-place variant: modifies k (and v); slots >= n_keep keep their content."""
    kept_idx = np.ascontiguousarray(kept_idx, dtype=np.int32)
    n_streams, n_keep = kept_idx.shape
    n_src = k.shape[3] if n_src is None else int(n_src)
    lay = _layout_of(k)
    if v is not None:
        assert v.shape == k.shape and v.strides == k.strides and v.dtype == k.dtype
    _check(lib().sirllm_ref_compact_kv_inplace(_ptr(k), _ptr(v), C.byref(lay), n_src, _ptr(kept_idx),
                                               max(n_keep, 1), n_streams, n_keep), "compact_kv_inplace")
    return k, v


def step(logits: np.ndarray, token_ids: np.ndarray, vocab: int, held_scores: np.ndarray, n_new: int, policy,
         k_src: np.ndarray, v_src: np.ndarray):
    """One turn.  logits [n_streams*n_new, ld]; held_scores [n_streams, n_held]; k_src/v_src
    [streams, layers, heads, >= n_cand, head_dim] with the new tokens' K/V already at slots
    [n_held, n_cand).  Returns dict(new_scores, kept_idx, scores_out, k, v, evicted); when
    nothing is evicted k/v are the first n_cand slots of the inputs (the cache is unchanged)."""
    held_scores = np.ascontiguousarray(held_scores, dtype=np.float32)
    n_streams, n_held = held_scores.shape
    n_cand = n_held + n_new
    n_keep = n_keep_of(n_cand, policy)
    evicted = n_cand > n_keep
    tok = np.ascontiguousarray(token_ids, dtype=np.int32)
    assert logits.shape[0] == n_streams * n_new and tok.shape == (n_streams * n_new,)
    assert k_src.shape[3] >= n_cand
    E = np.full((n_streams, max(n_cand, 1)), np.nan, dtype=np.float32)
    E[:, :n_held] = held_scores
    kept = np.full((n_streams, max(n_keep, 1)), -1, dtype=np.int32)
    out = np.full((n_streams, max(n_keep, 1)), np.nan, dtype=np.float32)
    shape = k_src.shape[:3] + (n_keep,) + k_src.shape[4:]
    k_dst = np.zeros(shape, dtype=k_src.dtype)
    v_dst = np.zeros(shape, dtype=v_src.dtype)
    ls, ld_ = _layout_of(k_src), _layout_of(k_dst)
    assert v_src.shape == k_src.shape and v_src.strides == k_src.strides
    cp = _cpolicy(policy)
    _check(lib().sirllm_ref_step(_ptr(logits), _logits_dtype(logits), int(vocab), logits.shape[1], _ptr(tok),
                                 _ptr(E), E.shape[1], n_streams, n_held, n_new, C.byref(cp),
                                 _ptr(k_src), _ptr(v_src), C.byref(ls), _ptr(k_dst), _ptr(v_dst), C.byref(ld_),
                                 _ptr(kept), kept.shape[1], _ptr(out), out.shape[1]), "step")
    if not evicted:
        k_dst = k_src[:, :, :, :n_cand].copy()
        v_dst = v_src[:, :, :, :n_cand].copy()
    return dict(new_scores=E[:, n_held:n_cand].copy(), kept_idx=kept[:, :n_keep], scores_out=out[:, :n_keep],
                k=k_dst, v=v_dst, evicted=evicted)


def step_ragged(logits: np.ndarray, token_ids: np.ndarray, vocab: int, scores: np.ndarray, n_held, n_new, policy,
                k: np.ndarray, v: np.ndarray | None):
    """Ragged batch, in place: stream s has n_held[s] cached slots and n_new[s] new tokens (its logits rows
    follow those of stream s-1).  Each stream goes through the same pinned pieces as a uniform step:
    score -> append -> decay held -> select -> compact in place.  Modifies scores (new scores appended) and
    k / v; returns (kept_idx list, scores_out list, n_keep list)."""
    n_streams = scores.shape[0]
    tok = np.ascontiguousarray(token_ids, dtype=np.int32)
    budget = int(policy.n_sink) + int(policy.n_topk) + int(policy.n_recent)
    kept_all, out_all, keep_n = [], [], []
    r0 = 0
    for s in range(n_streams):
        h, n = int(n_held[s]), int(n_new[s])
        if n:
            scores[s, h:h + n] = score(np.ascontiguousarray(logits[r0:r0 + n]), tok[r0:r0 + n], vocab=vocab)
        r0 += n
        if h + n == 0:
            kept_all.append(np.zeros(0, np.int32)); out_all.append(np.zeros(0, np.float32)); keep_n.append(0)
            continue
        ki, so = decay_select(scores[s:s + 1, :h + n], h, n, policy)
        if h + n > budget:
            compact_kv_inplace(k[s:s + 1], None if v is None else v[s:s + 1], ki, n_src=h + n)
        kept_all.append(ki[0]); out_all.append(so[0]); keep_n.append(ki.shape[1])
    return kept_all, out_all, keep_n
