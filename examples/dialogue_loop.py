"""A multi-turn loop over RetentiveCache (needs an MI355X and the built library).

Every turn brings n_new tokens: their K/V rows are written behind the live slots, the tokens are scored --
from stored logits (`step`) or straight from hidden states and the output embedding matrix
(`step_from_hidden`) -- the held scores decay, and the cache is compacted to sink + top-k + recent
(paper Alg. 1).  The script tracks which original token ended up in which slot and prints what survives.

    python examples/dialogue_loop.py [--turns 6] [--from-hidden]
"""
import argparse
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--turns", type=int, default=6)
    ap.add_argument("--from-hidden", action="store_true", help="score from hidden states and the LM head")
    args = ap.parse_args(argv)

    import torch
    from paper_2405_12528_amd import synth
    from paper_2405_12528_amd.cache import RetentiveCache

    if not torch.cuda.is_available():
        sys.exit("this example needs a GPU")
    dev = "cuda:0"
    w = synth.WORKLOADS["tiny"]                         # 64 tokens per turn, budget 32 = 4 sink + 20 top-k + 8 recent
    policy = (w.n_sink, w.n_topk, w.n_recent, w.decay)
    cache = RetentiveCache(1, w.n_layers, w.n_kv_heads, w.head_dim, policy, max_new=w.n_new,
                           kv_dtype=torch.float32, device=dev)
    origin = torch.zeros((0, 2), dtype=torch.int64)     # (turn, token) of every live slot, tracked on the host
    for turn in range(1, args.turns + 1):
        k_new, v_new = cache.new_kv_slots(w.n_new)
        k_new.copy_(synth.make_kv(w, n_pos=w.n_new, turn=turn, device=dev, which="k"))
        v_new.copy_(synth.make_kv(w, n_pos=w.n_new, turn=turn, device=dev, which="v"))
        tok = synth.make_token_ids(w, turn=turn, device=dev)
        if args.from_hidden:
            hidden, weight = synth.make_lmhead(w, turn=turn, device=dev)
            evicted = cache.step_from_hidden(hidden, weight, tok)
        else:
            evicted = cache.step(synth.make_logits(w, turn=turn, device=dev), tok, w.vocab)
        torch.cuda.synchronize()
        cand = torch.cat([origin, torch.stack([torch.full((w.n_new,), turn), torch.arange(w.n_new)], dim=1)])
        kept = cache.kept_idx[0, :cache.n_held].cpu().long()
        origin = cand[kept]
        per_turn = {t: int((origin[:, 0] == t).sum()) for t in range(1, turn + 1)}
        print(f"turn {turn}: {'evicted to' if evicted else 'holds'} {cache.n_held} slots; survivors per turn {per_turn}; "
              f"highest held score {cache.scores[0, :cache.n_held].max().item():.3f}")
    assert origin[:w.n_sink].tolist() == [[1, i] for i in range(w.n_sink)], "the sinks are the dialogue's first tokens"
    return origin


if __name__ == "__main__":
    main()
