"""Run by test_gpu_tuning.py in a process of its own with SIRLLM_TUNE=1: every launch-shape override the
library reads (workgroup size, vectors per lane, column parts, cached or non-temporal accesses, fused or
separate selection) must leave the results where the oracle puts them.  Prints one line per knob setting."""
import os
import sys

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))
from helpers import to_np                                   # noqa: E402
from oracle import ref                                      # noqa: E402
from paper_2405_12528_amd import binding as b, synth        # noqa: E402

DEV = "cuda:0"
KNOBS = ("SIRLLM_SCORE_BLOCK", "SIRLLM_SCORE_NT", "SIRLLM_GATHER_BLOCK", "SIRLLM_GATHER_UNROLL", "SIRLLM_GATHER_NT",
         "SIRLLM_FUSE_SELECT", "SIRLLM_INPLACE_BLOCK", "SIRLLM_INPLACE_UNROLL", "SIRLLM_INPLACE_PARTS",
         "SIRLLM_INPLACE_NT", "SIRLLM_INPLACE_TICKET", "SIRLLM_GATHER_SCALAR_IDX", "SIRLLM_GATHER_ROTATE", "SIRLLM_LMHEAD_WIDE")


def set_knobs(**kw):
    for k in KNOBS:
        os.environ.pop(k, None)
    for k, v in kw.items():
        os.environ["SIRLLM_" + k] = str(v)
    return " ".join(f"{k}={v}" for k, v in kw.items()) or "defaults"


def close(gpu, want):
    err = np.abs(gpu.astype(np.float64) - want.astype(np.float64))
    return bool((err <= 1e-6 + 1e-5 * np.abs(want)).all())


def check_score(label):
    for dtype, V in ((torch.float32, 70001), (torch.bfloat16, 32000), (torch.float16, 5003)):
        g = torch.Generator().manual_seed(V)
        z = (torch.randn((7, V), generator=g) * 3).to(dtype).to(DEV)
        tok = torch.randint(0, V, (7,), generator=g, dtype=torch.int32).to(DEV)
        out = torch.zeros(7, device=DEV)
        b.sirllm_score(z, tok, out)
        torch.cuda.synchronize()
        assert close(to_np(out), ref.score(to_np(z), to_np(tok))), f"score {dtype} under {label}"


def kv_pair(S, L, H, P, D, dtype):
    mod = 32749
    k = (synth.tagged_kv(S, L, H, P, D, 0) % mod).to(dtype).to(DEV)
    v = (synth.tagged_kv(S, L, H, P, D, 1) % mod).to(dtype).to(DEV)
    return k, v


def kept_list(rng, S, P, n_keep):
    kept = np.stack([np.sort(rng.choice(P, n_keep, replace=False)) for _ in range(S)]).astype(np.int32)
    kept[:, :4] = np.arange(4)
    kept = np.sort(kept, axis=1)
    for s in range(S):
        if len(np.unique(kept[s])) != n_keep:
            kept[s] = np.sort(rng.choice(P, n_keep, replace=False))
    return kept


def check_gather(label):
    rng = np.random.default_rng(5)
    for (S, L, H, P, D, dtype, n_keep) in ((2, 3, 2, 2300, 128, torch.bfloat16, 1111), (1, 2, 2, 700, 100, torch.bfloat16, 300),
                                           (1, 1, 2, 90, 7, torch.int16, 41)):
        k, v = kv_pair(S, L, H, P, D, dtype)
        kept = kept_list(rng, S, P, n_keep)
        kd = torch.full((S, L, H, n_keep + 1, D), 77, dtype=dtype, device=DEV)
        vd = torch.full_like(kd, 77)
        b.sirllm_compact_kv(k, v, kd, vd, torch.from_numpy(kept).to(DEV), n_keep)
        torch.cuda.synchronize()
        rk, rv = ref.compact_kv(to_np(k), to_np(v), kept)
        assert np.array_equal(to_np(kd)[:, :, :, :n_keep], rk) and np.array_equal(to_np(vd)[:, :, :, :n_keep], rv), \
            f"gather {P}x{D} under {label}"
        assert bool((kd[:, :, :, n_keep:] == 77).all())


def check_inplace(label, scratch=False):
    rng = np.random.default_rng(6)
    for (S, L, H, P, D, dtype, n_keep) in ((2, 2, 2, 9000, 128, torch.bfloat16, 4500), (1, 1, 2, 4300, 128, torch.bfloat16, 4100),
                                           (1, 2, 2, 700, 100, torch.bfloat16, 300), (1, 1, 2, 90, 7, torch.int16, 41)):
        k, v = kv_pair(S, L, H, P, D, dtype)
        kept = kept_list(rng, S, P, n_keep)
        hk, hv = to_np(k).copy(), to_np(v).copy()
        ref.compact_kv_inplace(hk, hv, kept)
        ws = torch.full((b.SIRLLM_INPLACE_WORKSPACE_BYTES,), 0x33, dtype=torch.uint8, device=DEV) if scratch else None
        b.sirllm_compact_kv_inplace(k, v, torch.from_numpy(kept).to(DEV), n_keep, workspace=ws)
        torch.cuda.synchronize()
        assert np.array_equal(to_np(k), hk) and np.array_equal(to_np(v), hv), f"in-place {P}x{D} under {label}"


def check_step(label):
    for n_held, n_new, pol in ((200, 30, (4, 100, 40, 0.9)), (200, 30, (4, 100, 10, 0.9))):    # new within / beyond the recent window
        S, V, n_cand = 2, 777, n_held + n_new
        g = torch.Generator().manual_seed(n_held + pol[2])
        z = (torch.randn((S * n_new, V), generator=g) * 2).to(DEV)
        tok = torch.randint(0, V, (S * n_new,), generator=g, dtype=torch.int32).to(DEV)
        scores = torch.zeros((S, n_cand), device=DEV)
        scores[:, :n_held] = (torch.rand((S, n_held), generator=g) * 6).to(DEV)
        held = to_np(scores[:, :n_held]).copy()
        k, v = kv_pair(S, 2, 2, n_cand, 16, torch.float32)
        P = b.Policy(*pol)
        n_keep = min(n_cand, pol[0] + pol[1] + pol[2])
        kd = torch.zeros((S, 2, 2, n_keep, 16), device=DEV); vd = torch.zeros_like(kd)
        kept = torch.zeros((S, n_keep), dtype=torch.int32, device=DEV); so = torch.zeros((S, n_keep), device=DEV)
        b.sirllm_step(z, tok, V, scores, n_held, n_new, P, k, v, kd, vd, kept, so)
        torch.cuda.synchronize()
        new = to_np(scores[:, n_held:])
        assert close(new.reshape(-1), ref.score(to_np(z), to_np(tok))), f"step scores under {label}"
        cand = np.concatenate([held, new], axis=1)              # teacher-forced: the oracle selects on the GPU's scores
        r_idx, r_sc = ref.decay_select(cand, n_held, n_new, ref.Policy(*pol))
        assert np.array_equal(to_np(kept), r_idx) and np.array_equal(to_np(so), r_sc), f"step selection under {label}"
        rk, rv = ref.compact_kv(to_np(k), to_np(v), r_idx)
        assert np.array_equal(to_np(kd), rk) and np.array_equal(to_np(vd), rv), f"step K/V under {label}"


def check_lmhead(label):
    for n, d, V in ((54, 256, 3000), (7, 128, 66000), (100, 192, 700), (64, 96, 500), (90, 64, 66000), (200, 128, 900)):      # every tile shape that has two stage widths
        g = torch.Generator(device=DEV).manual_seed(n + V)
        h = (torch.randn((n, d), generator=g, device=DEV) + 0.5).to(torch.bfloat16)
        w = (torch.randn((V, d), generator=g, device=DEV) * (3.0 / d ** 0.5)).to(torch.bfloat16)
        tok = torch.randint(0, V, (n,), generator=g, device=DEV, dtype=torch.int32)
        out = torch.zeros(n, device=DEV)
        ws = torch.empty(b.sirllm_lmhead_workspace_bytes(n, V), dtype=torch.uint8, device=DEV)
        b.sirllm_lmhead_score(h, w, tok, out, ws)
        torch.cuda.synchronize()
        want = ref.lmhead_score(to_np(h), to_np(w), to_np(tok))
        err = np.abs(to_np(out).astype(np.float64) - want)
        assert bool((err <= 2e-5 + 1e-5 * np.abs(want)).all()), f"lmhead {n}x{d}x{V} under {label}"


def main():
    assert os.environ.get("SIRLLM_TUNE"), "run with SIRLLM_TUNE=1"
    assert torch.cuda.is_available()
    n = 0
    for blk in (256, 512, 1024):
        for nt in (0, 1):
            label = set_knobs(SCORE_BLOCK=blk, SCORE_NT=nt)
            check_score(label); check_step(label); n += 1
            print("ok", label, flush=True)
    for blk in (64, 128, 256, 512):
        for un in (1, 2):
            for nt in (0, 1):
                label = set_knobs(GATHER_BLOCK=blk, GATHER_UNROLL=un, GATHER_NT=nt)
                check_gather(label); n += 1
                print("ok", label, flush=True)
    for blk in (64, 128):                                      # rows of 256 bytes: scalar or per-lane indices, tiles exchanged or not
        for scalar in (0, 1):
            for rot in (0, 1):
                label = set_knobs(GATHER_BLOCK=blk, GATHER_SCALAR_IDX=scalar, GATHER_ROTATE=rot)
                check_gather(label); n += 1
                print("ok", label, flush=True)
    for wide in (0, 1):                                        # LM-head tiles for up to 128 rows: stages of 32 or of 64 K elements
        label = set_knobs(LMHEAD_WIDE=wide)
        check_lmhead(label); n += 1
        print("ok", label, flush=True)
    for fuse in (0, 1):
        label = set_knobs(FUSE_SELECT=fuse)
        check_step(label); n += 1
        print("ok", label, flush=True)
    for blk in (256, 512, 1024):
        for un in (2, 4, 8):
            for parts, nt in ((1, 1), (2, 1), (4, 0), (1, 0)):
                label = set_knobs(INPLACE_BLOCK=blk, INPLACE_UNROLL=un, INPLACE_PARTS=parts, INPLACE_NT=nt, INPLACE_TICKET=(blk // 256 + un) % 2)
                check_inplace(label, scratch=True)
                check_inplace(label); n += 1
                print("ok", label, flush=True)
    for t in (0, 1):                                           # a workspace is given; ticket order forced off / on at any size
        label = set_knobs(INPLACE_TICKET=t)
        check_inplace(label, scratch=True); n += 1
        print("ok", label, flush=True)
    label = set_knobs()
    check_score(label); check_gather(label); check_inplace(label); check_inplace(label, scratch=True); check_step(label)
    print(f"ALL OK: {n} override settings", flush=True)


if __name__ == "__main__":
    main()
