"""Shared test plumbing: torch <-> numpy views that keep the exact bytes."""
import numpy as np
import torch


def to_np(t: torch.Tensor) -> np.ndarray:
    """Host numpy view/copy with identical bytes; bfloat16 comes back as uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def bf16_bits_to_f64(a: np.ndarray) -> np.ndarray:
    return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def logits_f64(a: np.ndarray) -> np.ndarray:
    """Exact widening to float64: uint16 = bfloat16 bit patterns, float16 / float32 by numpy's own conversion."""
    return bf16_bits_to_f64(a) if a.dtype == np.uint16 else a.astype(np.float64)


def read_golden(path):
    out = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = line.split("=")
            vals = [int(x) for x in v.split()]
            out[k.strip()] = vals[0] if len(vals) == 1 else vals
    return out
