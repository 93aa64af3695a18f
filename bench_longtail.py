#!/usr/bin/env python3
"""The 20000-sequence long-tail batch (config 4: 32 / 8 heads, head_dim 128, ChunkSize 16384) end to end on one GPU.

The batch is planned whole by cf_build_chunks (about 1100 chunks, 17.7 M tokens).  Its activations (Q, O, dO, dQ:
145 GB each) do not fit one GPU at once, so the dependency groups are placed and run a few at a time, as a
training loop would see them: each round places as many groups as fit a token budget, runs their forward and
backward passes (section 4.2 order inside every group) and frees them.  Only the attention calls are timed (HIP
events around each round's forward + backward); placing a round (allocation, drawing the synthetic values on the
device, building the descriptors) is outside the timed region, inputs are resident when it starts.

Prints one JSON line: total attention time, TFLOP/s over the unmasked pairs of the WHOLE batch, rounds.

    python bench_longtail.py [--tokens-per-round 1500000]
"""
import argparse
import json
import os
import sys
import time

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--tokens-per-round", type=int, default=1_500_000)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--max-rounds", type=int, default=0, help="stop after this many rounds (0: the whole batch)")
    ap.add_argument("--merge-tails", action="store_true", help="plan with CF_PLAN_MERGE_TAILS: the last, partial slice of a "
                    "split sequence shares a chunk with short sequences")
    args = ap.parse_args()

    import torch
    from paper_2503_02356_amd import binding as B
    from paper_2503_02356_amd import inputs
    from paper_2503_02356_amd.runner import ChunkAttention

    if not torch.cuda.is_available():
        sys.exit("bench_longtail.py: no GPU visible")
    cfg = inputs.CONFIGS["longtail_16k"]
    Hq, Hkv, D = cfg["Hq"], cfg["Hkv"], cfg["D"]
    lens, C = inputs.seq_lens("longtail_16k", args.seed, None)
    t0 = time.perf_counter()
    plan = B.cf_build_chunks_ex(lens, C, B.CF_PLAN_MERGE_TAILS) if args.merge_tails else B.cf_build_chunks(lens, C)
    plan_ms = (time.perf_counter() - t0) * 1e3
    vals = lambda sid, L: inputs.seq_values_device(args.seed, sid, int(lens[sid]), Hq, Hkv, D, cfg["dtype"], "cuda:0")

    # rounds: consecutive groups (plan order) up to the token budget
    group_tokens = [sum(int(plan.chunk_tokens[c]) for c in plan.group(g)) for g in range(plan.n_groups)]
    rounds, cur, cur_tokens = [], [], 0
    for g, n in enumerate(group_tokens):
        if cur and cur_tokens + n > args.tokens_per_round:
            rounds.append(cur)
            cur, cur_tokens = [], 0
        cur.append(g)
        cur_tokens += n
    if cur:
        rounds.append(cur)
    if args.max_rounds:
        rounds = rounds[:args.max_rounds]

    total_ms, total_pairs, total_tokens, per_round = 0.0, 0, 0, []
    for r, groups in enumerate(rounds):
        eng = ChunkAttention(plan, Hq, Hkv, D, cfg["dtype"], only_groups=groups).load(vals)
        if r == 0:                      # one untimed pass so that the first round does not pay for lazy initialisation
            eng.zero_grads(); eng.run_forward(); eng.run_backward()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        eng.zero_grads()
        eng.run_forward()
        eng.run_backward()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        tokens = sum(group_tokens[g] for g in groups)
        per_round.append({"groups": len(groups), "tokens": tokens, "ms": ms,
                          "tflops": 14.0 * D * Hq * eng.total_pairs / (ms * 1e-3) / 1e12})
        total_ms += ms
        total_pairs += eng.total_pairs
        total_tokens += tokens
        print(f"round {r + 1}/{len(rounds)}: {len(groups)} groups, {tokens} tokens, {ms:.1f} ms, "
              f"{per_round[-1]['tflops']:.0f} TFLOP/s", file=sys.stderr, flush=True)
        del eng
        torch.cuda.empty_cache()
    flop = 14.0 * D * Hq * total_pairs
    print(json.dumps({"metric": "chunk attention fwd+bwd TFLOP/s (unmasked pairs)", "value": flop / (total_ms * 1e-3) / 1e12,
                      "unit": "TFLOP/s", "attention_ms": total_ms, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": "config4_longtail_16k", "n_q_heads": Hq, "n_kv_heads": Hkv, "head_dim": D,
                                 "chunk_size": C, "n_sequences": int(len(lens)), "n_chunks": int(plan.n_chunks),
                                 "tokens": total_tokens, "unmasked_pairs": int(total_pairs), "flop": flop,
                                 "plan_build_ms": plan_ms, "rounds": len(rounds),
                                 "tokens_per_round": args.tokens_per_round, "merge_tails": args.merge_tails,
                                 "seed": args.seed},
                      "pct_of_bf16_mfma_peak": 100.0 * flop / (total_ms * 1e-3) / 1e12 / 2516.6,
                      "per_round": per_round}), flush=True)


if __name__ == "__main__":
    main()
