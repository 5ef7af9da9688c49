"""Thin ctypes binding of libsirllm.so: the entry points of include/sirllm.h under the same names.

Argument marshalling only -- device tensors come in as ``torch.Tensor`` (PyTorch supplies device
memory and the stream), go out as raw pointers, sizes and strides; every step of the path runs in
the library's HIP kernels.  There is no fallback: importing this module without a built library
raises, and a non-zero status from the library raises ``SirllmError``.
"""
from __future__ import annotations

import ctypes as C
import os
from collections import namedtuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsirllm.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it first (python -m paper_2405_12528_amd.build, or "
        "__graft_entry__.build()).  There is no CPU or PyTorch fallback for the retention step.")

_lib = C.CDLL(LIB_PATH)

SIRLLM_OK, SIRLLM_ERR_INVALID_ARG, SIRLLM_ERR_UNSUPPORTED, SIRLLM_ERR_WORKSPACE, SIRLLM_ERR_HIP = 0, -1, -2, -3, -4
SIRLLM_F32, SIRLLM_BF16, SIRLLM_F16 = 0, 1, 2
SIRLLM_MAX_CAND = 16777216
SIRLLM_SINGLE_WG_CAND = 32768

Policy = namedtuple("Policy", "n_sink n_topk n_recent decay")


class sirllm_policy(C.Structure):
    _fields_ = [("n_sink", C.c_int32), ("n_topk", C.c_int32), ("n_recent", C.c_int32), ("decay", C.c_float)]


class sirllm_kv_layout(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("elem_bytes", C.c_int32), ("stride_stream", C.c_int64), ("stride_layer", C.c_int64),
                ("stride_head", C.c_int64), ("stride_pos", C.c_int64)]


SIRLLM_BASELINE_STREAM, SIRLLM_BASELINE_INTERVAL, SIRLLM_BASELINE_RANDOM = 0, 1, 2

SIRLLM_STATIC_SCRATCH_BYTES = 1048576
SIRLLM_INPLACE_WORKSPACE_BYTES = 256

EXPORTS = ("sirllm_score", "sirllm_decay_select", "sirllm_decay_select_static", "sirllm_compact_kv", "sirllm_compact_kv_layers",
           "sirllm_compact_kv_inplace_layers", "sirllm_step", "sirllm_score_select", "sirllm_baseline_select",
           "sirllm_compact_kv_inplace", "sirllm_step_ragged", "sirllm_step_ragged_out_of_place", "sirllm_score_partial",
           "sirllm_score_merge", "sirllm_lmhead_score", "sirllm_lmhead_workspace_bytes",
           "sirllm_step_lmhead", "sirllm_step_lmhead_workspace_bytes", "sirllm_step_lmhead_ragged",
           "sirllm_step_lmhead_ragged_out_of_place", "sirllm_step_lmhead_ragged_workspace_bytes", "sirllm_workspace_bytes", "sirllm_status_string", "sirllm_version")

_vp, _i32, _i64, _sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
_PP, _LP = C.POINTER(sirllm_policy), C.POINTER(sirllm_kv_layout)
_lib.sirllm_score.argtypes = [_vp, C.c_int, _i64, _i32, _i64, _vp, _vp, _vp, _sz, _vp]
_lib.sirllm_decay_select.argtypes = [_vp, _i64, _i32, _i32, _i32, _PP, _vp, _i64, _vp, _i64, _vp, _sz, _vp]
_lib.sirllm_decay_select_static.argtypes = [_vp, _i64, _i32, _i32, _i32, _PP, _vp, _i64, _vp, _i64, _vp]
_lib.sirllm_decay_select_static.restype = C.c_int
_lib.sirllm_compact_kv.argtypes = [_vp, _vp, _LP, _i32, _vp, _vp, _LP, _vp, _i64, _i32, _i32, _vp]
_lib.sirllm_compact_kv_layers.argtypes = [_vp, _vp, _LP, _i32, _vp, _vp, _LP, _vp, _i64, _i32, _i32, _vp]
_lib.sirllm_compact_kv_layers.restype = C.c_int
_lib.sirllm_compact_kv_inplace_layers.argtypes = [_vp, _vp, _LP, _i32, _vp, _i64, _i32, _i32, _vp, _sz, _vp]
_lib.sirllm_compact_kv_inplace_layers.restype = C.c_int
_lib.sirllm_step.argtypes = [_vp, C.c_int, _i32, _i64, _vp, _vp, _i64, _i32, _i32, _i32, _PP,
                             _vp, _vp, _LP, _vp, _vp, _LP, _vp, _i64, _vp, _i64, _vp, _sz, _vp]
_lib.sirllm_score_select.argtypes = [_vp, C.c_int, _i32, _i64, _vp, _vp, _i64, _i32, _i32, _i32, _PP,
                                     _vp, _i64, _vp, _i64, _vp, _sz, _vp]
_lib.sirllm_score_select.restype = C.c_int
_lib.sirllm_baseline_select.argtypes = [C.c_int, _i32, _i32, _PP, C.c_uint64, C.c_uint64, _vp, _i64,
                                        C.POINTER(C.c_int32), _vp, _sz, _vp]
_lib.sirllm_baseline_select.restype = C.c_int
_lib.sirllm_compact_kv_inplace.argtypes = [_vp, _vp, _LP, _i32, _vp, _i64, _i32, _i32, _vp, _sz, _vp]
_lib.sirllm_compact_kv_inplace.restype = C.c_int
_lib.sirllm_step_ragged.argtypes = [_vp, C.c_int, _i32, _i64, _vp, _vp, _i64, _i32, _vp, _vp, _i64, _i32, _i32, _PP,
                                    _vp, _vp, _LP, _vp, _i64, _vp, _i64, _vp, _vp, _sz, _vp]
_lib.sirllm_step_ragged.restype = C.c_int
_lib.sirllm_step_ragged_out_of_place.argtypes = [_vp, C.c_int, _i32, _i64, _vp, _vp, _i64, _i32, _vp, _vp, _i64, _i32, _i32, _PP,
                                                 _vp, _vp, _LP, _vp, _vp, _LP, _vp, _i64, _vp, _i64, _vp, _vp, _sz, _vp]
_lib.sirllm_step_ragged_out_of_place.restype = C.c_int
_lib.sirllm_score_partial.argtypes = [_vp, C.c_int, _i64, _i32, _i64, _i32, _vp, _vp, _vp]
_lib.sirllm_score_partial.restype = C.c_int
_lib.sirllm_score_merge.argtypes = [_vp, _i32, _i64, _i64, _vp, _vp]
_lib.sirllm_score_merge.restype = C.c_int
_lib.sirllm_lmhead_score.argtypes = [_vp, _i64, _vp, _i64, C.c_int, _i32, _i64, _i32, _vp, _vp, _vp, _sz, _vp]
_lib.sirllm_lmhead_score.restype = C.c_int
_lib.sirllm_lmhead_workspace_bytes.argtypes = [_i64, _i32]
_lib.sirllm_lmhead_workspace_bytes.restype = _sz
_lib.sirllm_step_lmhead.argtypes = [_vp, _i64, _vp, _i64, C.c_int, _i32, _i32, _vp, _vp, _i64, _i32, _i32, _i32, _PP,
                                    _vp, _vp, _LP, _vp, _vp, _LP, _vp, _i64, _vp, _i64, _vp, _sz, _vp]
_lib.sirllm_step_lmhead.restype = C.c_int
_lib.sirllm_step_lmhead_workspace_bytes.argtypes = [_i32, _i32, _i64, _i32]
_lib.sirllm_step_lmhead_workspace_bytes.restype = _sz
_lib.sirllm_step_lmhead_ragged.argtypes = [_vp, _i64, _vp, _i64, C.c_int, _i32, _i32, _vp, _vp, _i64, _i32, _vp, _vp, _i64,
                                           _i32, _i32, _PP, _vp, _vp, _LP, _vp, _i64, _vp, _i64, _vp, _vp, _sz, _vp]
_lib.sirllm_step_lmhead_ragged.restype = C.c_int
_lib.sirllm_step_lmhead_ragged_out_of_place.argtypes = [_vp, _i64, _vp, _i64, C.c_int, _i32, _i32, _vp, _vp, _i64, _i32, _vp, _vp,
                                                        _i64, _i32, _i32, _PP, _vp, _vp, _LP, _vp, _vp, _LP, _vp, _i64, _vp,
                                                        _i64, _vp, _vp, _sz, _vp]
_lib.sirllm_step_lmhead_ragged_out_of_place.restype = C.c_int
_lib.sirllm_step_lmhead_ragged_workspace_bytes.argtypes = [_i32, _i32, _i64, _i32]
_lib.sirllm_step_lmhead_ragged_workspace_bytes.restype = _sz
for _n in ("sirllm_score", "sirllm_decay_select", "sirllm_compact_kv", "sirllm_step"):
    getattr(_lib, _n).restype = C.c_int
_lib.sirllm_workspace_bytes.argtypes = [_i32, _i32, _i64, _i32]
_lib.sirllm_workspace_bytes.restype = _sz
_lib.sirllm_status_string.argtypes = [C.c_int]
_lib.sirllm_status_string.restype = C.c_char_p
_lib.sirllm_version.restype = C.c_char_p


class SirllmError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status}: {sirllm_status_string(status)}")


def raw():
    """The ctypes library handle, for callers that pass raw pointers themselves."""
    return _lib


def sirllm_status_string(status: int) -> str:
    return _lib.sirllm_status_string(int(status)).decode()


def sirllm_version() -> str:
    return _lib.sirllm_version().decode()


def sirllm_workspace_bytes(n_streams: int, n_cand: int, n_rows: int, vocab: int) -> int:
    return int(_lib.sirllm_workspace_bytes(n_streams, n_cand, n_rows, vocab))


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return SIRLLM_F32
    if t.dtype == torch.bfloat16:
        return SIRLLM_BF16
    if t.dtype == torch.float16:
        return SIRLLM_F16
    raise TypeError(f"logits dtype {t.dtype} not supported (float32, bfloat16 or float16)")


def _on_device(*ts):
    for t in ts:
        if t is not None and not t.is_cuda:
            raise ValueError("libsirllm takes device tensors only")


def _policy(p) -> sirllm_policy:
    return sirllm_policy(int(p.n_sink), int(p.n_topk), int(p.n_recent), float(p.decay))


def kv_layout(t: torch.Tensor) -> sirllm_kv_layout:
    """Layout struct of a [streams, layers, kv_heads, slots, head_dim] tensor (any strides, last axis contiguous)."""
    if t.dim() != 5:
        raise ValueError("K/V tensors are [streams, layers, kv_heads, slots, head_dim]")
    if t.shape[4] > 1 and t.stride(4) != 1:
        raise ValueError("head_dim must be contiguous")
    return sirllm_kv_layout(t.shape[1], t.shape[2], t.shape[4], t.element_size(),
                            t.stride(0), t.stride(1), t.stride(2), t.stride(3))


def _ws(workspace):
    if workspace is None:
        return None, 0
    return workspace.data_ptr(), workspace.numel() * workspace.element_size()


def _check(rc, where):
    if rc != SIRLLM_OK:
        raise SirllmError(rc, where)


def sirllm_score(logits: torch.Tensor, token_ids: torch.Tensor, scores_out: torch.Tensor, vocab: int | None = None,
                 workspace: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """scores_out[r] = logsumexp(logits[r, :vocab]) - logits[r, token_ids[r]];  logits is [n_rows, ld]."""
    _on_device(logits, token_ids, scores_out, workspace)
    if logits.dim() != 2 or (logits.shape[1] > 1 and logits.stride(1) != 1):
        raise ValueError("logits must be [n_rows, ld] with contiguous rows")
    n_rows = logits.shape[0]
    ld = logits.stride(0) if n_rows > 1 else logits.shape[1]
    vocab = logits.shape[1] if vocab is None else int(vocab)
    if token_ids.dtype != torch.int32 or scores_out.dtype != torch.float32:
        raise TypeError("token_ids must be int32 and scores_out float32")
    if token_ids.numel() < n_rows or scores_out.numel() < n_rows or not token_ids.is_contiguous() \
            or not scores_out.is_contiguous():
        raise ValueError("token_ids / scores_out must be contiguous with n_rows entries")
    wp, wb = _ws(workspace)
    _check(_lib.sirllm_score(_ptr(logits), _dtype_code(logits), n_rows, vocab, ld, _ptr(token_ids),
                             _ptr(scores_out), wp, wb, _stream(stream)), "sirllm_score")
    return scores_out


def sirllm_lmhead_workspace_bytes(n_rows: int, vocab: int) -> int:
    return int(_lib.sirllm_lmhead_workspace_bytes(n_rows, vocab))


def sirllm_lmhead_score(hidden: torch.Tensor, weight: torch.Tensor, token_ids: torch.Tensor, scores_out: torch.Tensor,
                        workspace: torch.Tensor, d_model: int | None = None, vocab: int | None = None,
                        stream=None) -> torch.Tensor:
    """scores_out[r] = logsumexp_v(z[r, :vocab]) - z[r, token_ids[r]] with z = hidden[:, :d_model] @ weight[:, :d_model].T,
    the logits never stored.  hidden is [n_rows, ld_h], weight [>= vocab, ld_w], bf16 or f16, rows contiguous."""
    _on_device(hidden, weight, token_ids, scores_out, workspace)
    for t in (hidden, weight):
        if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
            raise ValueError("hidden / weight must be 2-D with contiguous rows")
    if hidden.dtype != weight.dtype:
        raise TypeError("hidden and weight must have the same element type")
    n_rows = hidden.shape[0]
    d_model = min(hidden.shape[1], weight.shape[1]) if d_model is None else int(d_model)
    vocab = weight.shape[0] if vocab is None else int(vocab)
    if vocab > weight.shape[0] or d_model > hidden.shape[1] or d_model > weight.shape[1]:
        raise ValueError("vocab / d_model exceed the arrays")
    if token_ids.dtype != torch.int32 or scores_out.dtype != torch.float32:
        raise TypeError("token_ids must be int32 and scores_out float32")
    if token_ids.numel() < n_rows or scores_out.numel() < n_rows or not token_ids.is_contiguous() \
            or not scores_out.is_contiguous():
        raise ValueError("token_ids / scores_out must be contiguous with n_rows entries")
    wp, wb = _ws(workspace)
    _check(_lib.sirllm_lmhead_score(_ptr(hidden), _row_stride(hidden), _ptr(weight), _row_stride(weight),
                                    _dtype_code(hidden), d_model, n_rows, vocab, _ptr(token_ids), _ptr(scores_out),
                                    wp, wb, _stream(stream)), "sirllm_lmhead_score")
    return scores_out


def sirllm_decay_select(scores: torch.Tensor, n_held: int, n_new: int, policy, kept_idx: torch.Tensor,
                        scores_out: torch.Tensor, workspace: torch.Tensor | None = None, stream=None):
    """scores [n_streams, >= n_held+n_new] f32; kept_idx [n_streams, >= n_keep] i32; scores_out likewise f32."""
    _on_device(scores, kept_idx, scores_out, workspace)
    for t, dt in ((scores, torch.float32), (kept_idx, torch.int32), (scores_out, torch.float32)):
        if t.dim() != 2 or t.dtype != dt or (t.shape[1] > 1 and t.stride(1) != 1):
            raise ValueError("scores / kept_idx / scores_out must be 2-D with contiguous rows (f32 / i32 / f32)")
    n_streams = scores.shape[0]
    if kept_idx.shape[0] != n_streams or scores_out.shape[0] != n_streams:
        raise ValueError("one row per stream in every array")
    p = _policy(policy)
    wp, wb = _ws(workspace)
    _check(_lib.sirllm_decay_select(_ptr(scores), _row_stride(scores), n_streams, n_held, n_new, C.byref(p),
                                    _ptr(kept_idx), _row_stride(kept_idx), _ptr(scores_out), _row_stride(scores_out),
                                    wp, wb, _stream(stream)), "sirllm_decay_select")
    return kept_idx, scores_out


def sirllm_decay_select_static(scores: torch.Tensor, n_held: int, n_new: int, policy, kept_idx: torch.Tensor,
                               scores_out: torch.Tensor, stream=None):
    """sirllm_decay_select without a workspace: the library's static device scratch serves large caches."""
    _on_device(scores, kept_idx, scores_out)
    for t, dt in ((scores, torch.float32), (kept_idx, torch.int32), (scores_out, torch.float32)):
        if t.dim() != 2 or t.dtype != dt or (t.shape[1] > 1 and t.stride(1) != 1):
            raise ValueError("scores / kept_idx / scores_out must be 2-D with contiguous rows (f32 / i32 / f32)")
    n_streams = scores.shape[0]
    if kept_idx.shape[0] != n_streams or scores_out.shape[0] != n_streams:
        raise ValueError("one row per stream in every array")
    p = _policy(policy)
    _check(_lib.sirllm_decay_select_static(_ptr(scores), _row_stride(scores), n_streams, n_held, n_new, C.byref(p),
                                           _ptr(kept_idx), _row_stride(kept_idx), _ptr(scores_out),
                                           _row_stride(scores_out), _stream(stream)), "sirllm_decay_select_static")
    return kept_idx, scores_out


def sirllm_baseline_select(kind: int, n_cand: int, policy, kept_idx: torch.Tensor, seed: int = 0, turn: int = 0,
                           workspace: torch.Tensor | None = None, stream=None) -> int:
    """Kept slots of a score-free baseline policy for n_streams = kept_idx.shape[0] streams; returns n_keep.
    workspace: only the random policy above 32768 slots per stream needs one (sirllm_workspace_bytes)."""
    _on_device(kept_idx, workspace)
    if kept_idx.dim() != 2 or kept_idx.dtype != torch.int32 or (kept_idx.shape[1] > 1 and kept_idx.stride(1) != 1):
        raise ValueError("kept_idx must be [n_streams, >= n_keep] int32 with contiguous rows")
    p = _policy(policy)
    n_keep = C.c_int32(-1)
    _check(_lib.sirllm_baseline_select(int(kind), kept_idx.shape[0], int(n_cand), C.byref(p), int(seed), int(turn),
                                       _ptr(kept_idx), _row_stride(kept_idx), C.byref(n_keep), *_ws(workspace),
                                       _stream(stream)),
           "sirllm_baseline_select")
    return n_keep.value


def _row_stride(t: torch.Tensor) -> int:
    return t.stride(0) if t.shape[0] > 1 else max(t.shape[1], 1)


def sirllm_compact_kv(k_src: torch.Tensor, v_src, k_dst: torch.Tensor, v_dst, kept_idx: torch.Tensor,
                      n_keep: int, n_src: int | None = None, stream=None):
    """dst[s, l, h, j, :] = src[s, l, h, kept_idx[s, j], :] for j < n_keep, for K and (if given) V."""
    _on_device(k_src, v_src, k_dst, v_dst, kept_idx)
    if kept_idx.dim() != 2 or kept_idx.dtype != torch.int32 or (kept_idx.shape[1] > 1 and kept_idx.stride(1) != 1):
        raise ValueError("kept_idx must be [n_streams, >= n_keep] int32 with contiguous rows")
    ls, ld = kv_layout(k_src), kv_layout(k_dst)
    if v_src is not None:
        if kv_layout_tuple(v_src) != kv_layout_tuple(k_src) or kv_layout_tuple(v_dst) != kv_layout_tuple(k_dst):
            raise ValueError("K and V must share one layout")
    n_streams = k_src.shape[0]
    n_src = k_src.shape[3] if n_src is None else int(n_src)
    if k_dst.shape[3] < n_keep or k_src.shape[3] < n_src or kept_idx.shape[0] != n_streams \
            or k_dst.shape[0] != n_streams:
        raise ValueError("destination has fewer than n_keep slots, or stream counts differ")
    _check(_lib.sirllm_compact_kv(_ptr(k_src), _ptr(v_src), C.byref(ls), n_src, _ptr(k_dst), _ptr(v_dst),
                                  C.byref(ld), _ptr(kept_idx), _row_stride(kept_idx), n_streams, int(n_keep),
                                  _stream(stream)), "sirllm_compact_kv")
    return k_dst, v_dst


def layer_layout(t: torch.Tensor, n_layers: int) -> sirllm_kv_layout:
    """Layout struct of ONE layer's [streams, kv_heads, slots, head_dim] tensor (any strides, last axis contiguous)."""
    if t.dim() != 4:
        raise ValueError("per-layer K/V tensors are [streams, kv_heads, slots, head_dim]")
    if t.shape[3] > 1 and t.stride(3) != 1:
        raise ValueError("head_dim must be contiguous")
    return sirllm_kv_layout(n_layers, t.shape[1], t.shape[3], t.element_size(), t.stride(0), 0, t.stride(1), t.stride(2))


def sirllm_compact_kv_layers(k_src, v_src, k_dst, v_dst, kept_idx: torch.Tensor, n_keep: int, n_src: int | None = None,
                             stream=None):
    """sirllm_compact_kv for a cache held as one tensor per layer: k_src, v_src, k_dst, v_dst are sequences of
    [streams, kv_heads, slots, head_dim] tensors (v_src and v_dst may both be None); all layers of one side share
    shape, strides and dtype."""
    sides = [list(k_src), None if v_src is None else list(v_src), list(k_dst), None if v_dst is None else list(v_dst)]
    n_layers = len(sides[0])
    if (sides[1] is None) != (sides[3] is None) or any(x is not None and len(x) != n_layers for x in sides):
        raise ValueError("one tensor per layer on every side; V on both sides or on neither")
    _on_device(kept_idx, *[t for x in sides if x is not None for t in x])
    if kept_idx.dim() != 2 or kept_idx.dtype != torch.int32 or (kept_idx.shape[1] > 1 and kept_idx.stride(1) != 1):
        raise ValueError("kept_idx must be [n_streams, >= n_keep] int32 with contiguous rows")
    if n_layers == 0:
        return k_dst, v_dst

    def same(ts):
        first = (ts[0].shape, ts[0].stride(), ts[0].dtype)
        return all((t.shape, t.stride(), t.dtype) == first for t in ts)
    if not all(same(x) for x in sides if x is not None):
        raise ValueError("the layers of one side must share shape, strides and dtype")
    if sides[1] is not None and ((sides[1][0].shape, sides[1][0].stride()) != (sides[0][0].shape, sides[0][0].stride())
                                 or (sides[3][0].shape, sides[3][0].stride()) != (sides[2][0].shape, sides[2][0].stride())):
        raise ValueError("K and V must share one layout")
    ls, ld = layer_layout(sides[0][0], n_layers), layer_layout(sides[2][0], n_layers)
    n_streams = sides[0][0].shape[0]
    n_src = sides[0][0].shape[2] if n_src is None else int(n_src)
    if sides[2][0].shape[2] < n_keep or sides[0][0].shape[2] < n_src or kept_idx.shape[0] != n_streams \
            or sides[2][0].shape[0] != n_streams:
        raise ValueError("destination has fewer than n_keep slots, or stream counts differ")
    arrays = [None if x is None else (C.c_void_p * n_layers)(*[t.data_ptr() for t in x]) for x in sides]
    _check(_lib.sirllm_compact_kv_layers(arrays[0], arrays[1], C.byref(ls), n_src, arrays[2], arrays[3], C.byref(ld),
                                         _ptr(kept_idx), _row_stride(kept_idx), n_streams, int(n_keep), _stream(stream)),
           "sirllm_compact_kv_layers")
    return k_dst, v_dst


def sirllm_compact_kv_inplace_layers(k, v, kept_idx: torch.Tensor, n_keep: int, n_src: int | None = None,
                                     workspace: torch.Tensor | None = None, stream=None):
    """sirllm_compact_kv_inplace for a cache held as one [streams, kv_heads, slots, head_dim] tensor per layer: k and v
    (v may be None) are sequences of such tensors sharing shape, strides and dtype."""
    k = list(k)
    v = None if v is None else list(v)
    n_layers = len(k)
    if v is not None and len(v) != n_layers:
        raise ValueError("one K and one V tensor per layer")
    _on_device(kept_idx, workspace, *k, *(v or []))
    if kept_idx.dim() != 2 or kept_idx.dtype != torch.int32 or (kept_idx.shape[1] > 1 and kept_idx.stride(1) != 1):
        raise ValueError("kept_idx must be [n_streams, >= n_keep] int32 with contiguous rows")
    if n_layers == 0:
        return k, v
    first = (k[0].shape, k[0].stride(), k[0].dtype)
    if any((t.shape, t.stride(), t.dtype) != first for t in k + (v or [])):
        raise ValueError("all layers, K and V alike, must share shape, strides and dtype")
    lay = layer_layout(k[0], n_layers)
    n_src = k[0].shape[2] if n_src is None else int(n_src)
    if k[0].shape[2] < n_src or kept_idx.shape[0] != k[0].shape[0]:
        raise ValueError("cache has fewer than n_src slots, or stream counts differ")
    ka = (C.c_void_p * n_layers)(*[t.data_ptr() for t in k])
    va = None if v is None else (C.c_void_p * n_layers)(*[t.data_ptr() for t in v])
    wp, wb = _ws(workspace)
    _check(_lib.sirllm_compact_kv_inplace_layers(ka, va, C.byref(lay), n_src, _ptr(kept_idx), _row_stride(kept_idx),
                                                 k[0].shape[0], int(n_keep), wp, wb, _stream(stream)),
           "sirllm_compact_kv_inplace_layers")
    return k, v


def sirllm_compact_kv_inplace(k: torch.Tensor, v, kept_idx: torch.Tensor, n_keep: int, n_src: int | None = None,
                              workspace: torch.Tensor | None = None, stream=None):
    """k[s, l, h, j, :] = k[s, l, h, kept_idx[s, j], :] for j < n_keep, in place (kept_idx strictly ascending)."""
    _on_device(k, v, kept_idx, workspace)
    if kept_idx.dim() != 2 or kept_idx.dtype != torch.int32 or (kept_idx.shape[1] > 1 and kept_idx.stride(1) != 1):
        raise ValueError("kept_idx must be [n_streams, >= n_keep] int32 with contiguous rows")
    lay = kv_layout(k)
    if v is not None and kv_layout_tuple(v) != kv_layout_tuple(k):
        raise ValueError("K and V must share one layout")
    n_src = k.shape[3] if n_src is None else int(n_src)
    if k.shape[3] < n_src or kept_idx.shape[0] != k.shape[0]:
        raise ValueError("cache has fewer than n_src slots, or stream counts differ")
    wp, wb = _ws(workspace)
    _check(_lib.sirllm_compact_kv_inplace(_ptr(k), _ptr(v), C.byref(lay), n_src, _ptr(kept_idx),
                                          _row_stride(kept_idx), k.shape[0], int(n_keep), wp, wb, _stream(stream)),
           "sirllm_compact_kv_inplace")
    return k, v


def kv_layout_tuple(t):
    L = kv_layout(t)
    return tuple(getattr(L, f) for f, _ in sirllm_kv_layout._fields_)


def sirllm_score_select(logits: torch.Tensor, token_ids: torch.Tensor, vocab: int, scores: torch.Tensor, n_held: int,
                        n_new: int, policy, kept_idx: torch.Tensor, scores_out: torch.Tensor,
                        workspace: torch.Tensor | None = None, stream=None) -> int:
    """The step without its K/V movement: scores the new tokens, decays, selects; returns n_keep.  Shapes as in
    sirllm_step."""
    _on_device(logits, token_ids, scores, kept_idx, scores_out, workspace)
    n_streams = scores.shape[0]
    if logits.dim() != 2 or (logits.shape[1] > 1 and logits.stride(1) != 1):
        raise ValueError("logits must be [n_streams*n_new, ld] with contiguous rows")
    if logits.shape[0] != n_streams * n_new or token_ids.numel() != n_streams * n_new:
        raise ValueError("one logits row and one token id per new token")
    if token_ids.dtype != torch.int32 or not token_ids.is_contiguous():
        raise TypeError("token_ids must be contiguous int32")
    for t, dt in ((scores, torch.float32), (kept_idx, torch.int32), (scores_out, torch.float32)):
        if t.dim() != 2 or t.dtype != dt or (t.shape[1] > 1 and t.stride(1) != 1) or t.shape[0] != n_streams:
            raise ValueError("scores / kept_idx / scores_out must be [n_streams, n] with contiguous rows")
    ld = logits.stride(0) if logits.shape[0] > 1 else logits.shape[1]
    p = _policy(policy)
    wp, wb = _ws(workspace)
    dtc = _dtype_code(logits) if n_new > 0 else SIRLLM_F32
    _check(_lib.sirllm_score_select(_ptr(logits) if n_new else None, dtc, int(vocab), ld,
                                    _ptr(token_ids) if n_new else None, _ptr(scores), _row_stride(scores), n_streams,
                                    int(n_held), int(n_new), C.byref(p), _ptr(kept_idx), _row_stride(kept_idx),
                                    _ptr(scores_out), _row_stride(scores_out), wp, wb, _stream(stream)),
           "sirllm_score_select")
    return min(n_held + n_new, p.n_sink + p.n_topk + p.n_recent)


def sirllm_step(logits: torch.Tensor, token_ids: torch.Tensor, vocab: int, scores: torch.Tensor, n_held: int,
                n_new: int, policy, k_src: torch.Tensor, v_src: torch.Tensor, k_dst, v_dst,
                kept_idx: torch.Tensor, scores_out: torch.Tensor, workspace: torch.Tensor | None = None,
                stream=None) -> int:
    """One retention step for n_streams = scores.shape[0] streams; returns n_keep.

    logits [n_streams*n_new, ld]; scores [n_streams, >= n_cand] (held scores in, new scores written
    behind them); k_src/v_src [streams, layers, kv_heads, >= n_cand, head_dim]; k_dst/v_dst the same
    with >= n_keep slots (may be None when n_cand <= budget: nothing is evicted then)."""
    _on_device(logits, token_ids, scores, k_src, v_src, k_dst, v_dst, kept_idx, scores_out, workspace)
    n_streams = scores.shape[0]
    if logits.dim() != 2 or (logits.shape[1] > 1 and logits.stride(1) != 1):
        raise ValueError("logits must be [n_streams*n_new, ld] with contiguous rows")
    if logits.shape[0] != n_streams * n_new or token_ids.numel() != n_streams * n_new:
        raise ValueError("one logits row and one token id per new token")
    if token_ids.dtype != torch.int32 or not token_ids.is_contiguous():
        raise TypeError("token_ids must be contiguous int32")
    for t, dt in ((scores, torch.float32), (kept_idx, torch.int32), (scores_out, torch.float32)):
        if t.dim() != 2 or t.dtype != dt or (t.shape[1] > 1 and t.stride(1) != 1) or t.shape[0] != n_streams:
            raise ValueError("scores / kept_idx / scores_out must be [n_streams, n] with contiguous rows")
    ld = logits.stride(0) if logits.shape[0] > 1 else logits.shape[1]
    p = _policy(policy)
    n_cand = n_held + n_new
    budget = p.n_sink + p.n_topk + p.n_recent
    n_keep = min(n_cand, budget)
    ls = kv_layout(k_src)
    if kv_layout_tuple(v_src) != kv_layout_tuple(k_src):
        raise ValueError("K and V must share one layout")
    if k_src.shape[0] != n_streams or k_src.shape[3] < n_cand:
        raise ValueError("source cache must hold n_cand slots for every stream")
    if k_dst is not None:
        ldst = kv_layout(k_dst)
        if kv_layout_tuple(v_dst) != kv_layout_tuple(k_dst) or k_dst.shape[3] < n_keep or k_dst.shape[0] != n_streams:
            raise ValueError("destination cache must hold n_keep slots for every stream, K and V alike")
    else:
        ldst = ls
    wp, wb = _ws(workspace)
    _check(_lib.sirllm_step(_ptr(logits), _dtype_code(logits), int(vocab), ld, _ptr(token_ids),
                            _ptr(scores), _row_stride(scores), n_streams, n_held, n_new, C.byref(p),
                            _ptr(k_src), _ptr(v_src), C.byref(ls), _ptr(k_dst), _ptr(v_dst), C.byref(ldst),
                            _ptr(kept_idx), _row_stride(kept_idx), _ptr(scores_out), _row_stride(scores_out),
                            wp, wb, _stream(stream)), "sirllm_step")
    return n_keep


def sirllm_step_lmhead_workspace_bytes(n_streams: int, n_cand: int, n_rows: int, vocab: int) -> int:
    return int(_lib.sirllm_step_lmhead_workspace_bytes(n_streams, n_cand, n_rows, vocab))


def sirllm_step_lmhead(hidden: torch.Tensor, weight: torch.Tensor, token_ids: torch.Tensor, scores: torch.Tensor,
                       n_held: int, n_new: int, policy, k_src: torch.Tensor, v_src: torch.Tensor, k_dst, v_dst,
                       kept_idx: torch.Tensor, scores_out: torch.Tensor, workspace: torch.Tensor,
                       d_model: int | None = None, vocab: int | None = None, stream=None) -> int:
    """sirllm_step with the scores taken from hidden [n_streams*n_new, ld_h] and weight [>= vocab, ld_w] (bf16 or
    f16) instead of stored logits; returns n_keep."""
    _on_device(hidden, weight, token_ids, scores, k_src, v_src, k_dst, v_dst, kept_idx, scores_out, workspace)
    n_streams = scores.shape[0]
    for t in (hidden, weight):
        if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
            raise ValueError("hidden / weight must be 2-D with contiguous rows")
    if hidden.dtype != weight.dtype:
        raise TypeError("hidden and weight must have the same element type")
    if hidden.shape[0] != n_streams * n_new or token_ids.numel() != n_streams * n_new:
        raise ValueError("one hidden-state row and one token id per new token")
    if token_ids.dtype != torch.int32 or not token_ids.is_contiguous():
        raise TypeError("token_ids must be contiguous int32")
    for t, dt in ((scores, torch.float32), (kept_idx, torch.int32), (scores_out, torch.float32)):
        if t.dim() != 2 or t.dtype != dt or (t.shape[1] > 1 and t.stride(1) != 1) or t.shape[0] != n_streams:
            raise ValueError("scores / kept_idx / scores_out must be [n_streams, n] with contiguous rows")
    d_model = min(hidden.shape[1], weight.shape[1]) if d_model is None else int(d_model)
    vocab = weight.shape[0] if vocab is None else int(vocab)
    if vocab > weight.shape[0] or d_model > hidden.shape[1] or d_model > weight.shape[1]:
        raise ValueError("vocab / d_model exceed the arrays")
    p = _policy(policy)
    n_cand = n_held + n_new
    n_keep = min(n_cand, p.n_sink + p.n_topk + p.n_recent)
    ls = kv_layout(k_src)
    if kv_layout_tuple(v_src) != kv_layout_tuple(k_src):
        raise ValueError("K and V must share one layout")
    if k_src.shape[0] != n_streams or k_src.shape[3] < n_cand:
        raise ValueError("source cache must hold n_cand slots for every stream")
    if k_dst is not None:
        ldst = kv_layout(k_dst)
        if kv_layout_tuple(v_dst) != kv_layout_tuple(k_dst) or k_dst.shape[3] < n_keep or k_dst.shape[0] != n_streams:
            raise ValueError("destination cache must hold n_keep slots for every stream, K and V alike")
    else:
        ldst = ls
    wp, wb = _ws(workspace)
    _check(_lib.sirllm_step_lmhead(_ptr(hidden), _row_stride(hidden), _ptr(weight), _row_stride(weight),
                                   _dtype_code(hidden), d_model, vocab, _ptr(token_ids),
                                   _ptr(scores), _row_stride(scores), n_streams, n_held, n_new, C.byref(p),
                                   _ptr(k_src), _ptr(v_src), C.byref(ls), _ptr(k_dst), _ptr(v_dst), C.byref(ldst),
                                   _ptr(kept_idx), _row_stride(kept_idx), _ptr(scores_out), _row_stride(scores_out),
                                   wp, wb, _stream(stream)), "sirllm_step_lmhead")
    return n_keep


def sirllm_step_ragged(logits: torch.Tensor, token_ids: torch.Tensor, vocab: int, scores: torch.Tensor,
                       n_held: torch.Tensor, cu_new: torch.Tensor, total_new: int, max_cand: int, policy,
                       k: torch.Tensor, v, kept_idx: torch.Tensor, scores_out: torch.Tensor,
                       n_keep_out: torch.Tensor, max_new: int | None = None, workspace: torch.Tensor | None = None,
                       stream=None) -> None:
    """Ragged in-place step: per-stream sizes in the device int32 arrays n_held [S] and cu_new [S+1];
    max_cand / max_new are host upper bounds of n_held[s] + n_new[s] and n_new[s] (max_new defaults to
    min(total_new, max_cand), which is always a valid bound)."""
    _on_device(logits, token_ids, scores, n_held, cu_new, k, v, kept_idx, scores_out, n_keep_out, workspace)
    n_streams = scores.shape[0]
    for t, n in ((n_held, n_streams), (cu_new, n_streams + 1), (n_keep_out, n_streams)):
        if t.dtype != torch.int32 or t.dim() != 1 or t.numel() != n or not t.is_contiguous():
            raise ValueError("n_held [S], cu_new [S+1], n_keep_out [S] must be contiguous int32 device vectors")
    if logits.dim() != 2 or (logits.shape[1] > 1 and logits.stride(1) != 1) or logits.shape[0] != total_new:
        raise ValueError("logits must be [total_new, ld] with contiguous rows")
    if token_ids.dtype != torch.int32 or not token_ids.is_contiguous() or token_ids.numel() != total_new:
        raise TypeError("token_ids must be contiguous int32 with total_new entries")
    for t, dt in ((scores, torch.float32), (kept_idx, torch.int32), (scores_out, torch.float32)):
        if t.dim() != 2 or t.dtype != dt or (t.shape[1] > 1 and t.stride(1) != 1) or t.shape[0] != n_streams:
            raise ValueError("scores / kept_idx / scores_out must be [n_streams, n] with contiguous rows")
    ld = logits.stride(0) if logits.shape[0] > 1 else logits.shape[1]
    lay = kv_layout(k)
    if v is not None and kv_layout_tuple(v) != kv_layout_tuple(k):
        raise ValueError("K and V must share one layout")
    if k.shape[0] != n_streams or k.shape[3] < max_cand:
        raise ValueError("the cache must hold max_cand slots for every stream")
    p = _policy(policy)
    wp, wb = _ws(workspace)
    dtc = _dtype_code(logits) if total_new > 0 else SIRLLM_F32
    _check(_lib.sirllm_step_ragged(_ptr(logits) if total_new else None, dtc, int(vocab), ld,
                                   _ptr(token_ids) if total_new else None, _ptr(scores), _row_stride(scores),
                                   n_streams, _ptr(n_held), _ptr(cu_new), int(total_new), int(max_cand),
                                   int(min(total_new, max_cand) if max_new is None else max_new), C.byref(p),
                                   _ptr(k), _ptr(v), C.byref(lay), _ptr(kept_idx), _row_stride(kept_idx),
                                   _ptr(scores_out), _row_stride(scores_out), _ptr(n_keep_out), wp, wb,
                                   _stream(stream)), "sirllm_step_ragged")


def sirllm_step_ragged_out_of_place(logits: torch.Tensor, token_ids: torch.Tensor, vocab: int, scores: torch.Tensor,
                                    n_held: torch.Tensor, cu_new: torch.Tensor, total_new: int, max_cand: int, policy,
                                    k_src: torch.Tensor, v_src, k_dst: torch.Tensor, v_dst, kept_idx: torch.Tensor,
                                    scores_out: torch.Tensor, n_keep_out: torch.Tensor, max_new: int | None = None,
                                    workspace: torch.Tensor | None = None, stream=None) -> None:
    """Ragged step that writes every accepted stream's kept slots from (k_src, v_src) into (k_dst, v_dst) -- compacted when
    the stream is over its budget, all of them otherwise -- and leaves a flagged stream's destination untouched; arguments
    otherwise as for sirllm_step_ragged."""
    _on_device(logits, token_ids, scores, n_held, cu_new, k_src, v_src, k_dst, v_dst, kept_idx, scores_out, n_keep_out, workspace)
    n_streams = scores.shape[0]
    for t, n in ((n_held, n_streams), (cu_new, n_streams + 1), (n_keep_out, n_streams)):
        if t.dtype != torch.int32 or t.dim() != 1 or t.numel() != n or not t.is_contiguous():
            raise ValueError("n_held [S], cu_new [S+1], n_keep_out [S] must be contiguous int32 device vectors")
    if logits.dim() != 2 or (logits.shape[1] > 1 and logits.stride(1) != 1) or logits.shape[0] != total_new:
        raise ValueError("logits must be [total_new, ld] with contiguous rows")
    if token_ids.dtype != torch.int32 or not token_ids.is_contiguous() or token_ids.numel() != total_new:
        raise TypeError("token_ids must be contiguous int32 with total_new entries")
    for t, dt in ((scores, torch.float32), (kept_idx, torch.int32), (scores_out, torch.float32)):
        if t.dim() != 2 or t.dtype != dt or (t.shape[1] > 1 and t.stride(1) != 1) or t.shape[0] != n_streams:
            raise ValueError("scores / kept_idx / scores_out must be [n_streams, n] with contiguous rows")
    ld = logits.stride(0) if logits.shape[0] > 1 else logits.shape[1]
    if (v_src is None) != (v_dst is None):
        raise ValueError("V on both sides or on neither")
    if v_src is not None and (kv_layout_tuple(v_src) != kv_layout_tuple(k_src) or kv_layout_tuple(v_dst) != kv_layout_tuple(k_dst)):
        raise ValueError("K and V must share one layout on each side")
    if k_src.shape[0] != n_streams or k_src.shape[3] < max_cand or k_dst.shape[0] != n_streams:
        raise ValueError("the source cache must hold max_cand slots for every stream")
    p = _policy(policy)
    if k_dst.shape[3] < min(max_cand, p.n_sink + p.n_topk + p.n_recent):
        raise ValueError("the destination cache must hold the budget for every stream")
    ls, ld_ = kv_layout(k_src), kv_layout(k_dst)
    wp, wb = _ws(workspace)
    dtc = _dtype_code(logits) if total_new > 0 else SIRLLM_F32
    _check(_lib.sirllm_step_ragged_out_of_place(
        _ptr(logits) if total_new else None, dtc, int(vocab), ld, _ptr(token_ids) if total_new else None, _ptr(scores),
        _row_stride(scores), n_streams, _ptr(n_held), _ptr(cu_new), int(total_new), int(max_cand),
        int(min(total_new, max_cand) if max_new is None else max_new), C.byref(p), _ptr(k_src), _ptr(v_src), C.byref(ls),
        _ptr(k_dst), _ptr(v_dst), C.byref(ld_), _ptr(kept_idx), _row_stride(kept_idx), _ptr(scores_out),
        _row_stride(scores_out), _ptr(n_keep_out), wp, wb, _stream(stream)), "sirllm_step_ragged_out_of_place")


def sirllm_step_lmhead_ragged_workspace_bytes(n_streams: int, max_cand: int, total_new: int, vocab: int) -> int:
    return int(_lib.sirllm_step_lmhead_ragged_workspace_bytes(n_streams, max_cand, total_new, vocab))


def sirllm_step_lmhead_ragged(hidden: torch.Tensor, weight: torch.Tensor, token_ids: torch.Tensor, scores: torch.Tensor,
                              n_held: torch.Tensor, cu_new: torch.Tensor, total_new: int, max_cand: int, policy,
                              k: torch.Tensor, v, kept_idx: torch.Tensor, scores_out: torch.Tensor,
                              n_keep_out: torch.Tensor, workspace: torch.Tensor, max_new: int | None = None,
                              d_model: int | None = None, vocab: int | None = None, stream=None) -> None:
    """sirllm_step_ragged with the scores taken from hidden [total_new, ld_h] and weight [>= vocab, ld_w] (bf16 or
    f16) instead of stored logits."""
    _on_device(hidden, weight, token_ids, scores, n_held, cu_new, k, v, kept_idx, scores_out, n_keep_out, workspace)
    n_streams = scores.shape[0]
    for t, n in ((n_held, n_streams), (cu_new, n_streams + 1), (n_keep_out, n_streams)):
        if t.dtype != torch.int32 or t.dim() != 1 or t.numel() != n or not t.is_contiguous():
            raise ValueError("n_held [S], cu_new [S+1], n_keep_out [S] must be contiguous int32 device vectors")
    for t in (hidden, weight):
        if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
            raise ValueError("hidden / weight must be 2-D with contiguous rows")
    if hidden.dtype != weight.dtype:
        raise TypeError("hidden and weight must have the same element type")
    if hidden.shape[0] != total_new or token_ids.numel() != total_new:
        raise ValueError("one hidden-state row and one token id per new token")
    if token_ids.dtype != torch.int32 or not token_ids.is_contiguous():
        raise TypeError("token_ids must be contiguous int32")
    for t, dt in ((scores, torch.float32), (kept_idx, torch.int32), (scores_out, torch.float32)):
        if t.dim() != 2 or t.dtype != dt or (t.shape[1] > 1 and t.stride(1) != 1) or t.shape[0] != n_streams:
            raise ValueError("scores / kept_idx / scores_out must be [n_streams, n] with contiguous rows")
    d_model = min(hidden.shape[1], weight.shape[1]) if d_model is None else int(d_model)
    vocab = weight.shape[0] if vocab is None else int(vocab)
    if vocab > weight.shape[0] or d_model > hidden.shape[1] or d_model > weight.shape[1]:
        raise ValueError("vocab / d_model exceed the arrays")
    lay = kv_layout(k)
    if v is not None and kv_layout_tuple(v) != kv_layout_tuple(k):
        raise ValueError("K and V must share one layout")
    if k.shape[0] != n_streams or k.shape[3] < max_cand:
        raise ValueError("the cache must hold max_cand slots for every stream")
    p = _policy(policy)
    wp, wb = _ws(workspace)
    _check(_lib.sirllm_step_lmhead_ragged(_ptr(hidden) if total_new else None, _row_stride(hidden), _ptr(weight),
                                          _row_stride(weight), _dtype_code(hidden), d_model, vocab,
                                          _ptr(token_ids) if total_new else None, _ptr(scores), _row_stride(scores),
                                          n_streams, _ptr(n_held), _ptr(cu_new), int(total_new), int(max_cand),
                                          int(min(total_new, max_cand) if max_new is None else max_new), C.byref(p),
                                          _ptr(k), _ptr(v), C.byref(lay), _ptr(kept_idx), _row_stride(kept_idx),
                                          _ptr(scores_out), _row_stride(scores_out), _ptr(n_keep_out), wp, wb,
                                          _stream(stream)), "sirllm_step_lmhead_ragged")


def sirllm_step_lmhead_ragged_out_of_place(hidden: torch.Tensor, weight: torch.Tensor, token_ids: torch.Tensor,
                                           scores: torch.Tensor, n_held: torch.Tensor, cu_new: torch.Tensor, total_new: int,
                                           max_cand: int, policy, k_src: torch.Tensor, v_src, k_dst: torch.Tensor, v_dst,
                                           kept_idx: torch.Tensor, scores_out: torch.Tensor, n_keep_out: torch.Tensor,
                                           workspace: torch.Tensor, max_new: int | None = None, d_model: int | None = None,
                                           vocab: int | None = None, stream=None) -> None:
    """sirllm_step_lmhead_ragged with every accepted stream's kept slots written from (k_src, v_src) into (k_dst, v_dst), as
    sirllm_step_ragged_out_of_place does."""
    _on_device(hidden, weight, token_ids, scores, n_held, cu_new, k_src, v_src, k_dst, v_dst, kept_idx, scores_out, n_keep_out,
               workspace)
    n_streams = scores.shape[0]
    for t, n in ((n_held, n_streams), (cu_new, n_streams + 1), (n_keep_out, n_streams)):
        if t.dtype != torch.int32 or t.dim() != 1 or t.numel() != n or not t.is_contiguous():
            raise ValueError("n_held [S], cu_new [S+1], n_keep_out [S] must be contiguous int32 device vectors")
    for t in (hidden, weight):
        if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
            raise ValueError("hidden / weight must be 2-D with contiguous rows")
    if hidden.dtype != weight.dtype:
        raise TypeError("hidden and weight must have the same element type")
    if hidden.shape[0] != total_new or token_ids.numel() != total_new:
        raise ValueError("one hidden-state row and one token id per new token")
    if token_ids.dtype != torch.int32 or not token_ids.is_contiguous():
        raise TypeError("token_ids must be contiguous int32")
    for t, dt in ((scores, torch.float32), (kept_idx, torch.int32), (scores_out, torch.float32)):
        if t.dim() != 2 or t.dtype != dt or (t.shape[1] > 1 and t.stride(1) != 1) or t.shape[0] != n_streams:
            raise ValueError("scores / kept_idx / scores_out must be [n_streams, n] with contiguous rows")
    d_model = min(hidden.shape[1], weight.shape[1]) if d_model is None else int(d_model)
    vocab = weight.shape[0] if vocab is None else int(vocab)
    if vocab > weight.shape[0] or d_model > hidden.shape[1] or d_model > weight.shape[1]:
        raise ValueError("vocab / d_model exceed the arrays")
    if (v_src is None) != (v_dst is None):
        raise ValueError("V on both sides or on neither")
    if v_src is not None and (kv_layout_tuple(v_src) != kv_layout_tuple(k_src) or kv_layout_tuple(v_dst) != kv_layout_tuple(k_dst)):
        raise ValueError("K and V must share one layout on each side")
    if k_src.shape[0] != n_streams or k_src.shape[3] < max_cand or k_dst.shape[0] != n_streams:
        raise ValueError("the source cache must hold max_cand slots for every stream")
    p = _policy(policy)
    if k_dst.shape[3] < min(max_cand, p.n_sink + p.n_topk + p.n_recent):
        raise ValueError("the destination cache must hold the budget for every stream")
    ls, ld_ = kv_layout(k_src), kv_layout(k_dst)
    wp, wb = _ws(workspace)
    _check(_lib.sirllm_step_lmhead_ragged_out_of_place(
        _ptr(hidden) if total_new else None, _row_stride(hidden), _ptr(weight), _row_stride(weight), _dtype_code(hidden),
        d_model, vocab, _ptr(token_ids) if total_new else None, _ptr(scores), _row_stride(scores), n_streams, _ptr(n_held),
        _ptr(cu_new), int(total_new), int(max_cand), int(min(total_new, max_cand) if max_new is None else max_new),
        C.byref(p), _ptr(k_src), _ptr(v_src), C.byref(ls), _ptr(k_dst), _ptr(v_dst), C.byref(ld_), _ptr(kept_idx),
        _row_stride(kept_idx), _ptr(scores_out), _row_stride(scores_out), _ptr(n_keep_out), wp, wb, _stream(stream)),
        "sirllm_step_lmhead_ragged_out_of_place")



def sirllm_score_partial(logits_chunk: torch.Tensor, v_begin: int, token_ids: torch.Tensor, partial: torch.Tensor,
                         stream=None) -> torch.Tensor:
    """(m, s, z_tok) per row for the vocabulary columns [v_begin, v_begin + logits_chunk.shape[1])."""
    _on_device(logits_chunk, token_ids, partial)
    if logits_chunk.dim() != 2 or (logits_chunk.shape[1] > 1 and logits_chunk.stride(1) != 1):
        raise ValueError("logits_chunk must be [n_rows, n_cols] with contiguous rows (a column slice is fine)")
    n_rows, n_cols = logits_chunk.shape
    ld = logits_chunk.stride(0) if n_rows > 1 else n_cols
    if partial.dtype != torch.float32 or not partial.is_contiguous() or partial.numel() < 3 * n_rows:
        raise ValueError("partial must be contiguous float32 with 3*n_rows entries")
    if token_ids.dtype != torch.int32 or not token_ids.is_contiguous() or token_ids.numel() < n_rows:
        raise TypeError("token_ids must be contiguous int32 with n_rows entries")
    _check(_lib.sirllm_score_partial(_ptr(logits_chunk), _dtype_code(logits_chunk), n_rows, n_cols, ld, int(v_begin),
                                     _ptr(token_ids), _ptr(partial), _stream(stream)), "sirllm_score_partial")
    return partial


def sirllm_score_merge(partials: torch.Tensor, n_rows: int, scores_out: torch.Tensor, stream=None) -> torch.Tensor:
    """partials is [n_parts, >= 3*n_rows] float32 (one row per chunk); writes scores_out[n_rows]."""
    _on_device(partials, scores_out)
    if partials.dim() != 2 or partials.dtype != torch.float32 or (partials.shape[1] > 1 and partials.stride(1) != 1):
        raise ValueError("partials must be [n_parts, >= 3*n_rows] float32 with contiguous rows")
    if scores_out.dtype != torch.float32 or not scores_out.is_contiguous() or scores_out.numel() < n_rows:
        raise ValueError("scores_out must be contiguous float32 with n_rows entries")
    _check(_lib.sirllm_score_merge(_ptr(partials), partials.shape[0], _row_stride(partials), int(n_rows),
                                   _ptr(scores_out), _stream(stream)), "sirllm_score_merge")
    return scores_out
