"""Seeded, bounded randomized parity sweep: 150 plans over random lengths (uniform, lognormal, tile-edge values),
chunk sizes, head counts and launch modes (Algorithm 2 with K kept chunks, whole-plan launches, merged tails, tile
tables on/off, one or two streams, the single-writer dK/dV mode), each compared element by element with the fp64
oracle's unsplit attention at the benchmark spec's tolerance.  Stops at the first mismatch and names the case."""
import numpy as np
import pytest

from paper_2503_02356_amd import binding as B
from tests import parity as P

pytestmark = pytest.mark.gpu
N_CASES = 150


def cases(seed):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < N_CASES:
        Hq, Hkv = [(4, 2), (8, 1), (7, 7), (6, 3), (28, 4), (14, 2)][int(rng.integers(0, 6))]
        C = int(rng.choice([64, 128, 192, 256, 320, 1000]))
        k = int(rng.integers(1, 9))
        kind = int(rng.integers(0, 3))
        if kind == 0:
            lens = rng.integers(1, 3 * C, size=k)
        elif kind == 1:
            lens = np.clip(np.rint(rng.lognormal(np.log(C / 3), 1.0, size=k)), 1, 6 * C)
        else:
            lens = rng.choice([1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, C - 1, C, C + 1, 2 * C, 2 * C + 1], size=k)
        lens = [int(x) for x in lens]
        if sum(lens) > 3000:
            continue
        mode = dict(K=[None, None, 1, 2][int(rng.integers(0, 4))], fused_launch=bool(rng.integers(0, 2)),
                    merge_tails=bool(rng.integers(0, 2)), tile_tables=bool(rng.integers(0, 2)),
                    n_streams=int(rng.choice([1, 1, 2])), flags=int(rng.choice([0, 0, B.CF_FLAG_DKV_SINGLE_WRITER])))
        if mode["K"] is not None:
            mode["fused_launch"] = False
        out.append((lens, C, Hq, Hkv, mode, int(rng.integers(0, 1 << 30))))
    return out


def test_randomized_plans_match_the_oracle():
    for n, (lens, C, Hq, Hkv, mode, seed) in enumerate(cases(20250302)):
        what = f"fuzz case {n}: lens {lens} C {C} heads {Hq}/{Hkv} {mode} seed {seed}"
        print(what, flush=True)
        got, _ = P.run_gpu(lens, C, Hq, Hkv, 128, "bf16", seed=seed, **mode)
        ref = P.run_oracle(lens, Hq, Hkv, 128, "bf16", seed=seed)
        P.check(got, ref, "bf16", what)
