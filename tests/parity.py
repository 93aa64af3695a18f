"""Helpers for the GPU parity tests: run a workload through the library and through the oracle."""
import numpy as np

from oracle import chunking as CK
from oracle.run_plan import run_unsplit
from paper_2503_02356_amd import binding as B
from paper_2503_02356_amd import inputs
from paper_2503_02356_amd.runner import ChunkAttention

# spec tolerances: (max-abs, relative L2) per tensor
TOL = {"bf16": (2e-2, 5e-3), "fp32": (1e-5, 1e-5)}
NAMES = ("o", "lse", "dq", "dk", "dv")


def oracle_count_chunks(lens, C):
    return len(CK.build_chunks(lens, C)[0])


def errors(got, ref):
    """Per tensor over all sequences: max |got-ref| and ||got-ref||_2 / ||ref||_2."""
    out = {}
    for name in NAMES:
        num = den = 0.0
        mx = 0.0
        for sid in ref:
            d = got[sid][name] - ref[sid][name]
            mx = max(mx, float(np.abs(d).max())) if d.size else mx
            num += float((d * d).sum())
            den += float((ref[sid][name] ** 2).sum())
        # a reference that is exactly zero (dQ of a one-token sequence) has no relative error;
        # the max-abs bound still applies to it
        out[name] = (mx, np.sqrt(num / den) if den > 0 else 0.0)
    return out


def check(got, ref, dtype, what=""):
    max_abs, rel = TOL[dtype]
    errs = errors(got, ref)
    for name, (mx, r) in errs.items():
        assert np.isfinite(mx) and mx <= max_abs and r <= rel, f"{what} {name}: max-abs {mx:.3e} rel-L2 {r:.3e}"
    return errs


def run_gpu(lens, C, Hq, Hkv, D, dtype, seed, flags=0, K=None, scale=None, fused_launch=False, n_streams=1,
            merge_tails=False, tile_tables=True):
    """Chunk-plan the lengths with the library, run forward+backward on the GPU, return per-sequence results."""
    plan = B.cf_build_chunks_ex(lens, C, B.CF_PLAN_MERGE_TAILS) if merge_tails else B.cf_build_chunks(lens, C)
    vals = lambda sid, L: inputs.seq_values(seed, sid, lens[sid], Hq, Hkv, D, dtype)
    eng = ChunkAttention(plan, Hq, Hkv, D, dtype, scale=scale, flags=flags, fused_launch=fused_launch,
                         n_streams=n_streams, tile_tables=tile_tables).load(vals)
    if K is None:
        eng.run_forward()
        eng.run_backward()
    else:
        eng.run_schedule(K)
    return eng.results(), eng


def run_oracle(lens, Hq, Hkv, D, dtype, seed, scale=None):
    seqs = {i: inputs.seq_values(seed, i, L, Hq, Hkv, D, dtype) for i, L in enumerate(lens)}
    s = scale if scale is not None else 1.0 / np.sqrt(D)
    return run_unsplit(seqs, np.float32(s))


_PYTEST_CONFIG = None


def set_pytest_config(config):
    global _PYTEST_CONFIG
    _PYTEST_CONFIG = config


def progress(*args):
    """A progress line that reaches the terminal while the test is still running (pytest's capture would hold it
    back until the test ends): minutes-long oracle comparisons stay visibly alive."""
    capman = _PYTEST_CONFIG.pluginmanager.getplugin("capturemanager") if _PYTEST_CONFIG is not None else None
    if capman is None:
        print(*args, flush=True)
        return
    with capman.global_and_fixture_disabled():
        print(*args, flush=True)
