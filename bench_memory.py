#!/usr/bin/env python3
"""Device memory of Algorithm 2 (paper section 4.2; table 5's trend) measured on the attention path.

One split sequence plus a few short ones runs through the executor that really discards (SlotExecutor: K
activation slots, a poisoned scratch slot, key/value state per group; inputs and results in pinned host memory)
for several (ChunkSize, K).  Prints one JSON line per pair: the allocator's peak over the run
(torch.cuda.max_memory_allocated minus what was allocated before), the executor's own account by kind, the
K * ChunkSize bound on kept activations from cf_schedule_stats, passes and re-forwards, and the wall time.

    python bench_memory.py [--seq-len 32768] [--chunk-sizes 2048,4096,8192] [--ks 1,2,4]
"""
import argparse
import json
import os
import sys
import time

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--seq-len", type=int, default=32768)
    ap.add_argument("--chunk-sizes", default="2048,4096,8192")
    ap.add_argument("--ks", default="1,2,4")
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()

    import torch
    from paper_2503_02356_amd import binding as B
    from paper_2503_02356_amd import inputs
    from paper_2503_02356_amd.executor import SlotExecutor
    from paper_2503_02356_amd.runner import schedule_memory

    if not torch.cuda.is_available():
        sys.exit("bench_memory.py: no GPU visible")
    Hq, Hkv, D = 28, 4, 128
    lens = [args.seq_len, 700, 1500, 300]
    cache = {}

    def vals(sid, L):
        if sid not in cache:
            cache[sid] = inputs.seq_values(args.seed, sid, lens[sid], Hq, Hkv, D, "bf16")
        return cache[sid]
    for C in [int(x) for x in args.chunk_sizes.split(",")]:
        for K in [int(x) for x in args.ks.split(",")]:
            plan = B.cf_build_chunks(lens, C)
            ex = SlotExecutor(plan, Hq, Hkv, D, "bf16", K).load(vals)
            torch.cuda.synchronize()
            torch.cuda.empty_cache()
            torch.cuda.reset_peak_memory_stats()
            base = torch.cuda.memory_allocated()
            t0 = time.perf_counter()
            ex.run()
            secs = time.perf_counter() - t0
            peak = torch.cuda.max_memory_allocated() - base
            account = ex.device_bytes()
            pred = schedule_memory(plan, K, Hq, Hkv, D)
            print(json.dumps({"chunk_size": C, "K": K, "n_chunks": plan.n_chunks, "n_forward": ex.n_forward,
                              "n_reforward": pred["n_reforward"], "peak_slots_in_use": ex.peak_slots,
                              "measured_peak_bytes": int(peak), "accounted_bytes": int(sum(account.values())),
                              "account": {k: int(v) for k, v in account.items()},
                              "kept_activation_bound_bytes": int(pred["kept_activation_bytes"]),
                              "k_times_chunk_tokens": K * C, "state_bytes": int(pred["state_bytes"]),
                              "seconds": round(secs, 3)}), flush=True)
            del ex
            plan.close()


if __name__ == "__main__":
    main()
