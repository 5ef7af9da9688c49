#!/usr/bin/env python3
"""Benchmark of the SirLLM retention step on one MI355X.

A "step" is one call of sirllm_step: score the new tokens, decay the held scores, select
sink + top-k + recent, compact every layer's K/V.  Inputs are seeded synthetic tensors already
resident in HBM when the timed region starts.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llama3_8b] [--no-cpu-baseline]

The headline measurement (value, ms_per_step, roofline, cpu_baseline) is the workload named by
--workload.  After it, outside its timed region, the default run also times the step on the other
workloads ("workloads" in the JSON line: min / median / max over repetitions) and three plain
streaming kernels ("ceilings": what this GPU gives a read-only scan, a fill and a copy of 1 GiB).
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0     # MI355X published HBM3E peak
OTHER_WORKLOADS = ("llama2_7b", "mistral_7b", "batched_dialogue", "rps_dialogue")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_launches(torch, fn, n, group=8):
    """Average, median and minimum duration (ms) of one launch: n groups of `group` back-to-back
    launches, each group bracketed by two events on the stream the kernels run on."""
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    for e0, e1 in evs:
        e0.record()
        for _ in range(group):
            fn()
        e1.record()
    torch.cuda.synchronize()
    ts = sorted(e0.elapsed_time(e1) / group for e0, e1 in evs)
    return sum(ts) / len(ts), ts[len(ts) // 2], ts[0]


class StepBench:
    """Inputs and outputs of one workload's step, resident in HBM, and the calls that are timed."""

    def __init__(self, torch, b, synth, w, dev):
        self.torch, self.b, self.w, self.dev = torch, b, w, dev
        S, n_held, n_new, n_cand, n_keep = w.n_streams, w.n_held, w.n_new, w.n_cand, w.n_keep
        self.pol = b.Policy(w.n_sink, w.n_topk, w.n_recent, w.decay)
        # Logits smaller than the 256 MB Infinity Cache would be served from it if one buffer were reused step
        # after step: rotate among enough distinct sets that at least 600 MB of logits pass between two uses of
        # the same set.  (The K/V sets are above 1.5 GB in every large workload and need no rotation.)
        logit_bytes = S * n_new * w.vocab * w.logit_bytes
        self.n_sets = 1 if logit_bytes >= 600e6 or w.name == "tiny" else min(32, -(-int(600e6) // logit_bytes))
        self.logit_sets = [synth.make_logits(w, turn=1 + i, device=dev) for i in range(self.n_sets)]
        self.tok_sets = [synth.make_token_ids(w, turn=1 + i, device=dev) for i in range(self.n_sets)]
        self.logit_bytes = logit_bytes
        self.scores = torch.zeros((S, n_cand), device=dev)
        self.scores[:, :n_held] = synth.make_held_scores(w, device=dev)
        self.k_src = synth.make_kv(w, device=dev, which="k")
        self.v_src = synth.make_kv(w, device=dev, which="v")
        dst_shape = (S, w.n_layers, w.n_kv_heads, n_keep, w.head_dim)
        self.k_dst = torch.zeros(dst_shape, dtype=self.k_src.dtype, device=dev)
        self.v_dst = torch.zeros(dst_shape, dtype=self.k_src.dtype, device=dev)
        self.kept = torch.zeros((S, n_keep), dtype=torch.int32, device=dev)
        self.scores_out = torch.zeros((S, n_keep), device=dev)
        self.new_scores = torch.zeros(S * n_new, device=dev)
        ws_bytes = b.sirllm_workspace_bytes(S, n_cand, S * n_new, w.vocab)
        self.ws = torch.zeros(max(ws_bytes, 256), dtype=torch.uint8, device=dev) if ws_bytes else None
        self.turn = 0
        torch.cuda.synchronize()

    def _next_set(self):
        i = self.turn % self.n_sets
        self.turn += 1
        return self.logit_sets[i], self.tok_sets[i]

    def step(self):
        w = self.w
        z, t = self._next_set()
        self.b.sirllm_step(z, t, w.vocab, self.scores, w.n_held, w.n_new, self.pol, self.k_src, self.v_src,
                           self.k_dst, self.v_dst, self.kept, self.scores_out, workspace=self.ws)

    def gather(self, kept=None):
        self.b.sirllm_compact_kv(self.k_src, self.v_src, self.k_dst, self.v_dst, self.kept if kept is None else kept,
                                 self.w.n_keep, n_src=self.w.n_cand)

    def score(self):
        z, t = self._next_set()
        self.b.sirllm_score(z, t, self.new_scores, vocab=self.w.vocab, workspace=self.ws)

    def select(self):
        self.b.sirllm_decay_select(self.scores, self.w.n_held, self.w.n_new, self.pol, self.kept, self.scores_out,
                                   workspace=self.ws)

    def time_steps(self, steps, warmup):
        """ms per step: `steps` back-to-back steps between two events, after `warmup` untimed ones."""
        torch = self.torch
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        ev0.record()
        for _ in range(steps):
            self.step()
        ev1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        return ev0.elapsed_time(ev1) / steps, wall_ms / steps


def measure_other_workload(torch, b, synth, name, dev, reps=5):
    """The step on one of the non-headline workloads: `reps` repetitions of a timed run of several steps; the
    spread between repetitions is part of the result."""
    w = synth.WORKLOADS[name]
    sb = StepBench(torch, b, synth, w, dev)
    # gigabytes were handed back to the driver just before (the previous workload's buffers): one repetition in five
    # came out 2-3 x slower right after that without a pause, always on the first workload measured here
    torch.cuda.synchronize()
    time.sleep(0.3)
    bytes_ = w.algorithmic_bytes()
    est_ms = max(bytes_["total"] / 6.0e12 * 1e3, 0.03)
    steps = int(max(4, min(60, 40.0 / est_ms)))                # about 40 ms of GPU time per repetition
    # the first repetition follows allocation and input generation: a whole repetition's worth of untimed steps first
    runs = sorted(sb.time_steps(steps, warmup=2 if i else max(10, steps))[0] for i in range(reps))
    med = runs[len(runs) // 2]
    g_avg, _, g_min = time_launches(torch, sb.gather, 4, group=8)
    out = {"ms_per_step": {"min": round(runs[0], 5), "median": round(med, 5), "max": round(runs[-1], 5)},
           "reps": reps, "steps_per_rep": steps, "algorithmic_bytes": bytes_["total"],
           "hbm_gbps": round(bytes_["total"] / (med * 1e-3) / 1e9, 1),
           "frac": round(bytes_["total"] / (med * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
           "frac_range": [round(bytes_["total"] / (runs[-1] * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                          round(bytes_["total"] / (runs[0] * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)],
           "tokens_per_s": round(w.n_streams * w.n_new / (med * 1e-3), 1),
           "gather_us": round(g_avg * 1e3, 2),
           "gather_gbps": round(bytes_["compact"] / (g_avg * 1e-3) / 1e9, 1),
           "config": {"n_streams": w.n_streams, "n_new": w.n_new, "n_cand": w.n_cand, "budget": w.budget, "vocab": w.vocab,
                      "logits_dtype": w.logits_dtype, "kv": f"{w.n_layers}x{w.n_kv_heads}x{w.head_dim} {w.kv_dtype}"}}
    log(f"[bench] {name}: {runs[0]*1e3:.1f} / {med*1e3:.1f} / {runs[-1]*1e3:.1f} us per step (min / median / max of {reps} x "
        f"{steps} steps) -> {out['hbm_gbps']:.0f} GB/s = {100*out['frac']:.1f} % of peak; gather alone {g_avg*1e3:.1f} us")
    del sb
    torch.cuda.empty_cache()
    return out


def measure_ceilings(torch, dev):
    """Plain streaming kernels over 1 GiB (libmembench.so): what the memory system gives a read-only scan, a fill
    and a copy with 16-byte non-temporal accesses, in this very run."""
    path = os.path.join(ROOT, "paper_2405_12528_amd", "libmembench.so")
    if not os.path.exists(path):
        log("[bench] libmembench.so is not built: no ceilings")
        return None
    mb = ctypes.CDLL(path)
    vp, sz = ctypes.c_void_p, ctypes.c_size_t
    mb.membench_read.argtypes = [vp, sz, vp, ctypes.c_int, vp]
    mb.membench_write.argtypes = [vp, sz, ctypes.c_int, vp]
    mb.membench_copy.argtypes = [vp, vp, sz, ctypes.c_int, vp]
    n = 1 << 30
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream().cuda_stream

    def must(rc):
        if rc != 0:
            raise RuntimeError(f"membench call failed with {rc}")

    by_threads = {}
    for threads in (64, 128, 512):
        r_avg, _, _ = time_launches(torch, lambda: must(mb.membench_read(src.data_ptr(), n, sink.data_ptr(), threads, stream)), 5, group=4)
        w_avg, _, _ = time_launches(torch, lambda: must(mb.membench_write(dst.data_ptr(), n, threads, stream)), 5, group=4)
        c_avg, _, _ = time_launches(torch, lambda: must(mb.membench_copy(dst.data_ptr(), src.data_ptr(), n, threads, stream)), 5, group=4)
        by_threads[threads] = {"read_gbps": round(n / (r_avg * 1e-3) / 1e9, 1), "write_gbps": round(n / (w_avg * 1e-3) / 1e9, 1),
                               "copy_gbps": round(2 * n / (c_avg * 1e-3) / 1e9, 1)}
        log(f"[bench] streaming kernels over 1 GiB, {threads}-thread workgroups: read {by_threads[threads]['read_gbps']:.0f} GB/s, "
            f"write {by_threads[threads]['write_gbps']:.0f} GB/s, copy {by_threads[threads]['copy_gbps']:.0f} GB/s (read + written)")
    out = {"bytes": n}
    for k in ("read_gbps", "write_gbps", "copy_gbps"):
        out[k] = max(v[k] for v in by_threads.values())
    out["by_workgroup_threads"] = {str(t): v for t, v in by_threads.items()}
    out["note"] = ("1 GiB, 16-byte non-temporal accesses; the best of 64-, 128- and 512-thread workgroups for each; "
                   "copy counts bytes read + bytes written")
    log(f"[bench] streaming ceilings over 1 GiB: read {out['read_gbps']:.0f} GB/s, write {out['write_gbps']:.0f} GB/s, "
        f"copy {out['copy_gbps']:.0f} GB/s (read + written)")
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama3_8b")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the 'workloads' and 'ceilings' records (the step on the four other workloads and the "
                         "plain streaming kernels), e.g. under a profiler")
    ap.add_argument("--ragged-inplace", action="store_true",
                    help="also time sirllm_step_ragged (per-stream sizes in device memory, in-place compaction) on "
                         "the same shapes; reported under 'ragged_inplace' in the JSON line")
    ap.add_argument("--cpu-threads", type=int, default=0, help="0 = min(16, host cores)")
    ap.add_argument("--graph", action="store_true",
                    help="also replay the step from a captured HIP graph (no per-launch host cost): the per-step "
                         "latency of small turns")
    ap.add_argument("--lmhead", action="store_true",
                    help="also time sirllm_lmhead_score (scores straight from bf16 hidden states and the output "
                         "embedding matrix, logits never stored) on the workload's rows")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (every stream, the whole step); --gpus must be 1. "
                 "Sharding across GPUs (by stream, or by KV head with a replicated selection) is described in the "
                 "design notes, not built.")

    import torch
    from paper_2405_12528_amd import binding as b
    from paper_2405_12528_amd import synth

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = synth.WORKLOADS[args.workload]
    S, n_held, n_new, n_cand, n_keep = w.n_streams, w.n_held, w.n_new, w.n_cand, w.n_keep
    log(f"[bench] {synth.describe(w)}")

    # ---- inputs, resident in HBM ---------------------------------------------------------
    sb = StepBench(torch, b, synth, w, dev)
    pol, scores, kept, scores_out, ws = sb.pol, sb.scores, sb.kept, sb.scores_out, sb.ws
    k_src, v_src, k_dst, v_dst, new_scores = sb.k_src, sb.v_src, sb.k_dst, sb.v_dst, sb.new_scores
    logits, tok = sb.logit_sets[0], sb.tok_sets[0]
    log(f"[bench] rotating among {sb.n_sets} logits set(s) of {sb.logit_bytes / 1e6:.1f} MB")

    # ---- the timed region: exactly K steps between two synchronisations ------------------
    ms_per_step, wall_ms_per_step = sb.time_steps(args.steps, args.warmup)
    log(f"[bench] {args.steps} steps: {ms_per_step * 1e3:.1f} us/step by events, {wall_ms_per_step * 1e3:.1f} us/step by host clock")

    bytes_ = w.algorithmic_bytes()
    tokens_per_s = S * n_new / (ms_per_step * 1e-3)
    step_gbps = bytes_["total"] / (ms_per_step * 1e-3) / 1e9

    # ---- the dominant kernel (the K/V gather), timed launch by launch with events on the
    #      stream it runs on, in the launch configuration the step uses ---------------------
    n_k = max(5, min(args.steps, 20))
    gather_avg, gather_med, gather_min = time_launches(torch, sb.gather, n_k)
    score_avg, score_med, score_min = time_launches(torch, sb.score, n_k)
    sel_avg, sel_med, sel_min = time_launches(torch, sb.select, n_k)
    log(f"[bench] per launch (avg/median/min us): gather {gather_avg*1e3:.1f}/{gather_med*1e3:.1f}/{gather_min*1e3:.1f}  "
        f"score {score_avg*1e3:.1f}/{score_med*1e3:.1f}/{score_min*1e3:.1f}  "
        f"decay_select {sel_avg*1e3:.1f}/{sel_med*1e3:.1f}/{sel_min*1e3:.1f}")
    # a plain copy of known size (1 GiB read + 1 GiB written) so that a counter run of this same
    # command holds its own calibration kernel for FETCH_SIZE / WRITE_SIZE
    calib_src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    calib_dst = torch.empty_like(calib_src)
    copy_avg, _, _ = time_launches(torch, lambda: calib_dst.copy_(calib_src), 3, group=2)
    copy_gbps = 2 * (1 << 30) / (copy_avg * 1e-3) / 1e9
    log(f"[bench] calibration copy of 1 GiB (torch's own kernel): {copy_avg*1e3:.1f} us -> {copy_gbps:.0f} GB/s")
    del calib_src, calib_dst
    # the same gather on the identity list 0..n_keep-1: a contiguous copy of the same size through the same kernel
    ident = torch.arange(n_keep, dtype=torch.int32, device=dev).repeat(S, 1).contiguous()
    ident_avg, _, _ = time_launches(torch, lambda: sb.gather(ident), max(3, n_k // 2))
    ident_gbps = bytes_["compact"] / (ident_avg * 1e-3) / 1e9
    sb.gather()                                                                        # leave the step's own result behind
    log(f"[bench] the gather on the identity list (contiguous copy, same kernel): {ident_avg*1e3:.1f} us -> {ident_gbps:.0f} GB/s")
    if bytes_["compact"] >= bytes_["score"]:
        # rows of 256 bytes are copied by a kernel of their own
        gather_name = "gather_rows16_kernel" if w.head_dim * w.kv_elem_bytes == 256 else "gather_rows_kernel"
        dom, dom_bytes, dom_ms = gather_name, bytes_["compact"], gather_avg
    else:
        dom, dom_bytes, dom_ms = "score_rows_kernel", bytes_["score"], score_avg
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9
    traffic, traffic_source = committed_traffic(dom, w.name)
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic, "traffic_source": traffic_source,
                "algorithmic_bytes_per_launch": dom_bytes, "avg_launch_us": round(dom_ms * 1e3, 2),
                "step": {"algorithmic_bytes": bytes_["total"], "achieved": round(step_gbps, 1),
                         "frac": round(step_gbps / HBM_PEAK_GBPS, 4)},
                "kernels_us": {"gather": round(gather_avg * 1e3, 2), "score": round(score_avg * 1e3, 2),
                               "decay_select": round(sel_avg * 1e3, 2)},
                "score_gbps": round(bytes_["score"] / (score_avg * 1e-3) / 1e9, 1),
                "calibration_copy_gbps": round(copy_gbps, 1), "identity_gather_gbps": round(ident_gbps, 1)}

    # ---- optional: the ragged in-place step on the same shapes --------------------------------
    ragged = None
    if args.ragged_inplace:
        held_dev = torch.full((S,), n_held, dtype=torch.int32, device=dev)
        cu_dev = torch.arange(0, (S + 1) * n_new, n_new, dtype=torch.int32, device=dev)
        keep_dev = torch.zeros(S, dtype=torch.int32, device=dev)

        # above 32768 slots per stream the selection's scratch is required; below, the workspace only carries the
        # in-place compaction's ticket and the step also runs without one
        large = n_cand > b.SIRLLM_SINGLE_WG_CAND
        ip_ws = torch.zeros(max(b.SIRLLM_INPLACE_WORKSPACE_BYTES, b.sirllm_workspace_bytes(S, n_cand, 0, 0)),
                            dtype=torch.uint8, device=dev)

        def ragged_step(scratch=ip_ws):      # repeated in place on the same buffers: the data changes, the traffic does not
            z, t = sb._next_set()
            b.sirllm_step_ragged(z, t, w.vocab, scores, held_dev, cu_dev, S * n_new, n_cand, pol,
                                 k_src, v_src, kept, scores_out, keep_dev, max_new=n_new, workspace=scratch)

        r_avg, r_med, r_min = time_launches(torch, ragged_step, n_k, group=4)
        ragged = {"ms_per_step": round(r_avg, 5), "hbm_gbps": round(bytes_["total"] / (r_avg * 1e-3) / 1e9, 1),
                  "frac": round(bytes_["total"] / (r_avg * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                  "vs_uniform_step": round(r_avg / ms_per_step, 4), "median_ms_per_step": round(r_med, 5)}
        rw_avg = r_avg if large else time_launches(torch, lambda: ragged_step(None), n_k, group=4)[0]
        ragged["ms_per_step_without_workspace"] = None if large else round(rw_avg, 5)
        for label, scratch in (("inplace_gather", ip_ws), ("inplace_gather_without_workspace", None)):
            ip_avg, _, _ = time_launches(
                torch, lambda: b.sirllm_compact_kv_inplace(k_src, v_src, kept, n_keep, n_src=n_cand, workspace=scratch), n_k, group=4)
            ragged[label + "_us"] = round(ip_avg * 1e3, 2)
            ragged[label + "_gbps"] = round(bytes_["compact"] / (ip_avg * 1e-3) / 1e9, 1)
        log(f"[bench] ragged in-place step: {r_avg*1e3:.1f} us -> {ragged['hbm_gbps']:.0f} GB/s ({rw_avg*1e3:.1f} us without a "
            f"workspace); in-place gather alone {ragged['inplace_gather_us']:.1f} us -> {ragged['inplace_gather_gbps']:.0f} GB/s "
            f"(planes by ticket), {ragged['inplace_gather_without_workspace_us']:.1f} us -> "
            f"{ragged['inplace_gather_without_workspace_gbps']:.0f} GB/s (planes by block index)")

        # the same ragged step with the K/V movement out of place (second buffer pair: the uniform step's k_dst / v_dst)
        def ragged_oop_step():
            z, t = sb._next_set()
            b.sirllm_step_ragged_out_of_place(z, t, w.vocab, scores, held_dev, cu_dev, S * n_new, n_cand, pol, k_src, v_src,
                                              k_dst, v_dst, kept, scores_out, keep_dev, max_new=n_new,
                                              workspace=ip_ws if large else None)

        o_avg, o_med, _ = time_launches(torch, ragged_oop_step, n_k, group=4)
        ragged["out_of_place_ms_per_step"] = round(o_avg, 5)
        ragged["out_of_place_median_ms_per_step"] = round(o_med, 5)
        ragged["out_of_place_vs_uniform_step"] = round(o_avg / ms_per_step, 4)
        log(f"[bench] ragged out-of-place step: {o_avg*1e3:.1f} us -> {bytes_['total'] / (o_avg * 1e-3) / 1e9:.0f} GB/s "
            f"(median of the timed groups: {o_med*1e3:.1f} us)")

    # ---- optional: the step replayed from a captured graph ----------------------------------------------
    graph_ms = None
    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            sb.step()                                    # warm-up on the capture stream
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        reps = 20
        hgraph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(hgraph):
            for _ in range(reps):                        # back-to-back steps in one graph, sets rotating as above
                sb.step()
        hgraph.replay()
        torch.cuda.synchronize()
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        g0.record()
        for _ in range(5):
            hgraph.replay()
        g1.record()
        torch.cuda.synchronize()
        graph_ms = g0.elapsed_time(g1) / (5 * reps)
        log(f"[bench] step replayed from a graph of {reps} steps: {graph_ms * 1e3:.1f} us/step")

    # ---- optional: scoring straight from the LM head (MFMA bound) ---------------------------------
    lmhead = None
    if args.lmhead:
        hid, wmat = synth.make_lmhead(w, turn=1, device=dev)
        # Inside a model step the embedding matrix is read once per step, behind gigabytes of other weights: it comes
        # from HBM, not from the 256 MB memory-side cache.  Rotate among enough copies of it to make that so here.
        w_bytes = wmat.numel() * wmat.element_size()
        n_w = min(8, max(2, -(-(3 << 29) // w_bytes)))
        wmats = [wmat] + [wmat.clone() for _ in range(n_w - 1)]
        turn_w = [0]

        def next_w():
            turn_w[0] = (turn_w[0] + 1) % n_w
            return wmats[turn_w[0]]

        log(f"[bench] LM head: rotating among {n_w} copies of the {w_bytes / 1e6:.0f} MB embedding matrix")
        lm_ws = torch.empty(b.sirllm_lmhead_workspace_bytes(hid.shape[0], w.vocab), dtype=torch.uint8, device=dev)
        lm_avg, lm_med, lm_min = time_launches(
            torch, lambda: b.sirllm_lmhead_score(hid, next_w(), tok, new_scores, lm_ws), n_k, group=2)
        flops = 2.0 * hid.shape[0] * w.vocab * w.d_model
        tfl = flops / (lm_avg * 1e-3) / 1e12
        lmhead = {"bound": "mfma", "kernel": "lmhead_score_kernel", "dtype": "bf16", "achieved": round(tfl, 1),
                  "peak": 2500.0, "unit": "TFLOP/s", "frac": round(tfl / 2500.0, 4), "ms": round(lm_avg, 4),
                  "rows": hid.shape[0], "vocab": w.vocab, "d_model": w.d_model,
                  "tokens_per_s": round(hid.shape[0] / (lm_avg * 1e-3), 1),
                  "logits_route_ms": round(score_avg, 4), "weight_copies": n_w}
        if hid.shape[0] <= 128:
            # up to 128 rows the matrix cores idle and the kernel streams the embedding matrix once: priced against HBM
            stream_gbps = (w.vocab * w.d_model + hid.shape[0] * w.d_model) * 2 / (lm_avg * 1e-3) / 1e9
            lmhead.update({"bound": "hbm", "achieved": round(stream_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                           "frac": round(stream_gbps / HBM_PEAK_GBPS, 4), "tflops": round(tfl, 1)})
        st_ws = torch.empty(max(b.sirllm_step_lmhead_workspace_bytes(S, n_cand, hid.shape[0], w.vocab), 256),
                            dtype=torch.uint8, device=dev)
        st_avg, _, _ = time_launches(
            torch, lambda: b.sirllm_step_lmhead(hid, next_w(), tok, scores, n_held, n_new, pol, k_src, v_src, k_dst, v_dst,
                                                kept, scores_out, st_ws), n_k, group=2)
        lmhead["step_ms"] = round(st_avg, 4)
        lmhead["step_tokens_per_s"] = round(hid.shape[0] / (st_avg * 1e-3), 1)
        log(f"[bench] step with the scores from the LM head: {st_avg*1e3:.1f} us")
        # context, not the product path: the same product by the library GEMM torch ships (logits stored in the hidden
        # states' type), alone and followed by this library's scan of those logits
        lib_logits = torch.empty((hid.shape[0], w.vocab), dtype=hid.dtype, device=dev)
        lib_scores = torch.empty(hid.shape[0], device=dev)
        mm_avg, _, _ = time_launches(torch, lambda: torch.mm(hid, next_w()[:w.vocab].t(), out=lib_logits), n_k, group=2)

        def library_route():
            torch.mm(hid, next_w()[:w.vocab].t(), out=lib_logits)
            b.sirllm_score(lib_logits, tok, lib_scores, vocab=w.vocab, workspace=ws)

        lr_avg, _, _ = time_launches(torch, library_route, n_k, group=2)
        lmhead["library_gemm_ms"] = round(mm_avg, 4)
        lmhead["library_gemm_tflops"] = round(flops / (mm_avg * 1e-3) / 1e12, 1)
        lmhead["library_gemm_then_scan_ms"] = round(lr_avg, 4)
        log(f"[bench] for comparison, torch.mm of the same operands (logits written out): {mm_avg*1e3:.1f} us -> "
            f"{lmhead['library_gemm_tflops']:.0f} TFLOP/s; followed by sirllm_score on them: {lr_avg*1e3:.1f} us")
        del lib_logits, lib_scores
        log(f"[bench] lmhead_score {hid.shape[0]} x {w.d_model} x {w.vocab}: {lm_avg*1e3:.1f}/{lm_med*1e3:.1f}/{lm_min*1e3:.1f} us "
            f"(avg/median/min) -> {tfl:.0f} TFLOP/s = {100 * tfl / 2500:.1f} % of 2.5 PFLOP/s"
            + (f"; the embedding matrix streamed at {lmhead['achieved']:.0f} GB/s = {100 * lmhead['frac']:.1f} % of 8 TB/s"
               if lmhead["bound"] == "hbm" else ""))
        del hid, wmat, wmats, lm_ws, st_ws

    # ---- the oracle on the host cores, same bytes, as a reported baseline ----------------
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(w, args, logits, tok, scores, k_src, v_src)

    out = {
        "metric": "entropy-scored tokens/sec + fused step HBM GB/s (% of MI355X peak)",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "vocab": w.vocab, "logits_dtype": w.logits_dtype, "n_streams": S,
                   "n_new": n_new, "n_cand": n_cand, "budget": w.budget, "n_sink": w.n_sink, "n_topk": w.n_topk,
                   "n_recent": w.n_recent, "decay": w.decay, "kv": f"{w.n_layers}x{w.n_kv_heads}x{w.head_dim} {w.kv_dtype}"},
        "step_hbm_gbps": round(step_gbps, 1), "step_pct_of_peak": round(100 * step_gbps / HBM_PEAK_GBPS, 2),
        "roofline": roofline, "cpu_baseline": cpu,
    }
    if ragged:
        out["ragged_inplace"] = ragged
    if lmhead:
        out["lmhead"] = lmhead
    if graph_ms is not None:
        out["graph_ms_per_step"] = round(graph_ms, 5)

    # ---- after the headline measurement: the other workloads and the streaming ceilings -------------
    if not args.no_other_workloads and args.workload == "llama3_8b":
        del sb, pol, scores, kept, scores_out, ws, k_src, v_src, k_dst, v_dst, new_scores, logits, tok, ident
        torch.cuda.empty_cache()
        out["ceilings"] = measure_ceilings(torch, dev)
        out["workloads"] = {name: measure_other_workload(torch, b, synth, name, dev) for name in OTHER_WORKLOADS}
    print(json.dumps(out), flush=True)


def committed_traffic(kernel, workload):
    """HBM bytes per launch of `kernel` as measured by the rocprofv3 FETCH_SIZE / WRITE_SIZE counter
    runs of this command, and the file that holds the figure: the committed summary under profiles/
    (a counter run cannot be made from inside the timed process).  (None, None) when no summary
    covers the workload."""
    import re
    rel = os.path.join("profiles", f"{kernel}__{workload}.md")
    try:
        m = re.search(r"^traffic_bytes_per_launch\s*=\s*(\d+)", open(os.path.join(ROOT, rel)).read(), flags=re.M)
    except OSError:
        return None, None
    return (int(m.group(1)), rel) if m else (None, None)


def cpu_baseline(w, args, logits, tok, scores, k_src, v_src):
    """The oracle's whole step on the host, on a bounded sample of the same workload: every new
    token of stream 0 (all of the workload when it has one stream)."""
    import numpy as np
    from oracle import ref

    def host(t):
        t = t.detach().cpu().contiguous()
        import torch
        return t.view(torch.int16).numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.numpy()

    threads = args.cpu_threads or min(16, os.cpu_count() or 1)
    threads = ref.set_threads(threads)
    n_new, n_held = w.n_new, w.n_held
    z = host(logits[:n_new])
    t = host(tok[:n_new])
    held = host(scores[:1, :n_held])
    k = host(k_src[:1])
    v = host(v_src[:1])
    pol = ref.Policy(w.n_sink, w.n_topk, w.n_recent, w.decay)
    ref.step(z, t, w.vocab, held, n_new, pol, k, v)                      # warm-up (page faults, thread pool)
    reps, t0 = 0, time.perf_counter()
    while True:
        ref.step(z, t, w.vocab, held, n_new, pol, k, v)
        reps += 1
        el = time.perf_counter() - t0
        if reps >= 3 or el > 20.0:
            break
    per = el / reps
    sample = (f"oracle sirllm_ref_step on stream 0 of {w.n_streams}: {n_new} tokens x V={w.vocab}, select over "
              f"{w.n_cand} slots, K/V gather of {w.n_keep} slots x {w.n_layers}x2x{w.n_kv_heads} planes; "
              f"{reps} repetitions after 1 warm-up")
    log(f"[bench] oracle: {per:.3f} s per stream-step on {threads} threads")
    out = {"value": round(n_new / per, 1), "unit": "tokens/s", "cores": threads, "kind": "oracle", "sample": sample,
           "seconds_per_stream_step": round(per, 4)}
    if threads > 1:                                    # the same once more on one thread (bounded: at most ~10 s)
        ref.set_threads(1)
        reps1, t1 = 0, time.perf_counter()
        while True:
            ref.step(z, t, w.vocab, held, n_new, pol, k, v)
            reps1 += 1
            el1 = time.perf_counter() - t1
            if reps1 >= 2 or el1 > 10.0:
                break
        ref.set_threads(threads)
        out["single_thread"] = {"value": round(n_new / (el1 / reps1), 1), "unit": "tokens/s", "cores": 1,
                                "seconds_per_stream_step": round(el1 / reps1, 4)}
        log(f"[bench] oracle: {el1 / reps1:.3f} s per stream-step on 1 thread")
    return out


if __name__ == "__main__":
    main()
