#!/usr/bin/env python3
"""(ChunkSize, K) sweep of the attention path alone, in the shape of the paper's table 6: one 262144-token
sequence plus short ones (the config-5 batch), chunked with several ChunkSize values while ChunkSize * K stays
constant, each run through Algorithm 2 (section 4.2) with that K.  What the table's end-to-end numbers mix
(kernel efficiency of small chunks, re-forward cost, pipeline bubbles) is reduced here to the first two:
there is no pipeline on one GPU.

Prints one JSON line per (ChunkSize, K): time of one Algorithm-2 step, TFLOP/s on the USEFUL work
(14 * D * Hq * unmasked pairs: re-forward passes cost time but add no useful FLOP), passes and re-forwards,
and the bytes section 4.2's schedule keeps (kept chunk activations, key/value state).

    python bench_sweep.py [--pairs 2048x16,8192x4,32768x1] [--steps 2]
"""
import argparse
import json
import os
import sys
import time

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--pairs", default="2048x16,8192x4,32768x1", help="comma list of ChunkSize x K")
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()

    import torch
    from paper_2503_02356_amd import binding as B
    from paper_2503_02356_amd import inputs
    from paper_2503_02356_amd.runner import ChunkAttention, schedule_memory

    if not torch.cuda.is_available():
        sys.exit("sweep_chunksize_k.py: no GPU visible")
    cfg = inputs.CONFIGS["long256k_32k"]
    Hq, Hkv, D = cfg["Hq"], cfg["Hkv"], cfg["D"]

    def count_chunks(lens, C):
        p = B.cf_build_chunks(lens, C)
        n = p.n_chunks
        p.close()
        return n
    # the batch itself (sequence lengths) is the config-5 one for every ChunkSize
    lens, _ = inputs.seq_lens("long256k_32k", args.seed, count_chunks)
    vals = lambda sid, L: inputs.seq_values_device(args.seed, sid, int(lens[sid]), Hq, Hkv, D, cfg["dtype"], "cuda:0")

    for item in args.pairs.split(","):
        C, K = (int(x) for x in item.lower().split("x"))
        plan = B.cf_build_chunks(lens, C)
        eng = ChunkAttention(plan, Hq, Hkv, D, cfg["dtype"]).load(vals)
        flop = 14.0 * D * Hq * eng.total_pairs

        def step():
            eng.zero_grads()
            eng.run_schedule(K)
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
        mem = schedule_memory(plan, K, Hq, Hkv, D)
        print(json.dumps({"chunk_size": C, "K": K, "n_chunks": int(plan.n_chunks), "ms_per_step": ms,
                          "useful_tflops": flop / (ms * 1e-3) / 1e12, "n_forward": mem["n_forward"],
                          "n_reforward": mem["n_reforward"], "n_backward": mem["n_backward"],
                          "peak_kept_tokens": mem["peak_kept_tokens"],
                          "kept_activation_GiB": mem["kept_activation_bytes"] / 2**30,
                          "state_GiB": mem["state_bytes"] / 2**30}), flush=True)
        del eng
        plan.close()
        torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
