"""Seeded synthetic inputs shared by the tests, the bench and the smoke check.

Holds no attention or chunking arithmetic: only random sequence lengths with the shape of the
paper's workloads (tables 1 and 2: a mass of short sequences with a thin, very long tail) and
N(0,1) tensor values.  The paper's datasets are not available; these stand in for them.
"""
import math

import numpy as np

# (name, dtype, n_q_heads, n_kv_heads, head_dim, chunk_size)
CONFIGS = {
    "tiny_fp32":      dict(dtype="fp32", Hq=1,  Hkv=1, D=64,  C=256),
    "packed_8k":      dict(dtype="bf16", Hq=28, Hkv=4, D=128, C=8192),
    "long32k_mixed":  dict(dtype="bf16", Hq=28, Hkv=4, D=128, C=8192),
    "longtail_16k":   dict(dtype="bf16", Hq=32, Hkv=8, D=128, C=16384),
    "long256k_32k":   dict(dtype="bf16", Hq=64, Hkv=8, D=128, C=32768),
}


def _lognormal_lengths(rng, n, mu, sigma, lo, hi):
    x = np.rint(rng.lognormal(mu, sigma, size=n))
    return np.clip(x, lo, hi).astype(np.int64)


def _fill_chunks(rng, count_chunks, C, n_chunks, mu, sigma, lo, hi, head=()):
    """Draw short lengths one at a time; keep them while the chunk builder still needs at most
    `n_chunks` packed chunks; stop at the first draw that would need one more."""
    lens = list(head)
    base = count_chunks(lens, C) if lens else 0
    while True:
        x = int(_lognormal_lengths(rng, 1, mu, sigma, lo, hi)[0])
        if count_chunks(lens + [x], C) - base > n_chunks:
            return lens
        lens.append(x)


def seq_lens(config, seed, count_chunks, scale_down=1):
    """Sequence lengths of one synthetic batch.

    count_chunks(lens, C) -> number of chunks the chunk builder makes (callback, so that this
    module stays free of the method).  scale_down divides chunk size and all length parameters
    (a structurally identical small instance).  Returns (lens int64 array, chunk_size).
    """
    rng = np.random.default_rng([seed, 0x5EED])
    sd = scale_down
    if config == "tiny_fp32":
        C = 256
        lens = list(rng.integers(8, 121, size=12)) + [700]
        return np.array(lens, dtype=np.int64), C
    if config == "packed_8k":
        C = 8192 // sd
        lens = _fill_chunks(rng, count_chunks, C, 16, math.log(600 / sd), 0.9, max(1, 16 // sd), C)
        return np.array(lens, dtype=np.int64), C
    if config == "long32k_mixed":
        C = 8192 // sd
        lens = _fill_chunks(rng, count_chunks, C, 8, math.log(600 / sd), 0.9, max(1, 16 // sd), C,
                            head=[32768 // sd])
        return np.array(lens, dtype=np.int64), C
    if config == "longtail_16k":
        C = 16384 // sd
        n = 20000 // sd
        n_long = max(1, round(0.0011 * n))
        sigma = 0.9
        mu = math.log(800 / sd) - sigma * sigma / 2          # lognormal mean 800
        short = _lognormal_lengths(rng, n - n_long, mu, sigma, max(1, 16 // sd), C)
        long_ = rng.integers(C + 1, 131072 // sd + 1, size=n_long)
        lens = np.concatenate([short, long_])
        rng.shuffle(lens)
        return lens.astype(np.int64), C
    if config == "long256k_32k":
        C = 32768 // sd
        lens = _fill_chunks(rng, count_chunks, C, 4, math.log(1000 / sd), 0.9, max(1, 16 // sd), C,
                            head=[262144 // sd])
        return np.array(lens, dtype=np.int64), C
    raise KeyError(config)


def round_to_bf16(x):
    """Round fp32 values to the nearest bf16 (ties to even), returned as fp32."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def seq_values(seed, seq_id, L, Hq, Hkv, D, dtype):
    """q, k, v, d_o of one sequence: i.i.d. N(0,1) fp32, rounded to bf16 values when dtype is
    'bf16'.  Each sequence has its own stream, so any one can be regenerated alone."""
    out = {}
    for t, (name, H) in enumerate((("q", Hq), ("k", Hkv), ("v", Hkv), ("d_o", Hq))):
        rng = np.random.default_rng([seed, int(seq_id), t, 0xA77])
        x = rng.standard_normal((int(L), H, D), dtype=np.float32)
        out[name] = round_to_bf16(x) if dtype == "bf16" else x
    return out


def seq_values_device(seed, seq_id, L, Hq, Hkv, D, dtype, device):
    """The same recipe drawn on the device by torch's seeded generator, for sizes where the host generator
    takes minutes (a 262144-token sequence of 64 heads is 19 GB of fp32): q, k, v, d_o as torch tensors in
    the storage dtype.  (A different stream than seq_values: the two are not interchangeable.)"""
    import torch
    out = {}
    for t, (name, H) in enumerate((("q", Hq), ("k", Hkv), ("v", Hkv), ("d_o", Hq))):
        g = torch.Generator(device=device)
        g.manual_seed((int(seed) * 1000003 + int(seq_id)) * 4 + t)
        x = torch.randn((int(L), H, D), generator=g, device=device, dtype=torch.float32)
        out[name] = x.to(torch.bfloat16) if dtype == "bf16" else x
    return out
