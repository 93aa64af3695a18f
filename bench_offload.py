#!/usr/bin/env python3
"""Cost and saving of key/value state offload (paper section 6.3's open optimisation) on the attention path: one
split sequence through several attention layers, once with every layer's key/value and gradient state resident on
the GPU and once with a window of two layers' state, the rest waiting in pinned host memory and prefetched while
the previous layer computes.  Prints one JSON line per mode: step time, device bytes held, bytes moved over the bus.

    python bench_offload.py [--seq-len 32768] [--chunk-size 8192] [--layers 8] [--windows 8,2]
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
    ap.add_argument("--chunk-size", type=int, default=8192)
    ap.add_argument("--layers", type=int, default=8)
    ap.add_argument("--windows", default=None, help="comma list of window sizes (default: layers, 2)")
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()

    import torch
    from paper_2503_02356_amd import inputs
    from paper_2503_02356_amd.offload import LayeredSequenceAttention

    if not torch.cuda.is_available():
        sys.exit("bench_offload.py: no GPU visible")
    Hq, Hkv, D = 28, 4, 128
    windows = [int(x) for x in args.windows.split(",")] if args.windows else [args.layers, 2]
    base = inputs.seq_values(args.seed, 0, args.seq_len, Hq, Hkv, D, "bf16")     # every layer reuses one draw, rolled
    pairs = args.seq_len * (args.seq_len + 1) // 2
    flop = 14.0 * D * Hq * pairs * args.layers
    for w in windows:
        torch.cuda.empty_cache()
        torch.cuda.reset_peak_memory_stats()
        before = torch.cuda.memory_allocated()
        eng = LayeredSequenceAttention(args.seq_len, args.chunk_size, args.layers, Hq, Hkv, D, w)
        eng.load(lambda layer: {k: v for k, v in base.items()})
        eng.run_step()                                         # warm-up
        t0 = time.perf_counter()
        for _ in range(args.steps):
            eng.run_step()
        secs = (time.perf_counter() - t0) / args.steps
        print(json.dumps({"window_layers": eng.window, "layers": args.layers, "offload": eng.offload,
                          "seq_len": args.seq_len, "chunk_size": args.chunk_size,
                          "ms_per_step": secs * 1e3, "tflops": flop / secs / 1e12,
                          "device_bytes_held": int(eng.device_bytes()),
                          "peak_allocated_bytes": int(torch.cuda.max_memory_allocated() - before),
                          "h2d_bytes_per_step": int(eng.h2d_bytes), "d2h_bytes_per_step": int(eng.d2h_bytes)}), flush=True)
        del eng


if __name__ == "__main__":
    main()
