"""Pins of oracle/pipeline.py: the bubble ratios the paper prints for its four-sequence pipeline example
(section 3.3, equation 1; section 4.3; section 5), closed forms, and conservation checks.  CPU only."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import chunking as CK
from oracle import pipeline as PL

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_pipeline_bubbles.txt")


def golden():
    rows = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if line:
            key, value = line.split("=")
            rows[key.strip()] = value.strip()
    return rows


def percent(fr, digits):
    return float(fr) * 100


def printed_as(fr, text):
    """True if the exact ratio prints as `text` percent either rounded or truncated to its digits (the paper
    truncates: it prints 3/7 as 42.8)."""
    digits = len(text.split(".")[1]) if "." in text else 0
    x = Fraction(fr) * 100 * 10 ** digits
    return text in (f"{int(x) / 10 ** digits:.{digits}f}", f"{round(float(fr) * 100, digits):.{digits}f}")


def test_paper_example_standard_1f1b():
    g = golden()
    r = PL.one_f_one_b([4, 2, 1, 1], 4)           # section 3.3: lengths 4, 2, 1, 1 Units on 4 stages
    assert r["bubble_ratio"] == Fraction(4, 7) and printed_as(r["bubble_ratio"], g["standard_1f1b_variable"])
    r = PL.one_f_one_b([2, 2, 2, 2], 4)           # "four sequences of equal length"
    assert r["bubble_ratio"] == Fraction(3, 7) and printed_as(r["bubble_ratio"], g["standard_1f1b_equal"])


def test_paper_example_state_aware_1f1b():
    g = golden()
    lens = [4, 2, 1, 1]
    chunks, groups = CK.build_chunks(lens, 2)      # section 4.3: ChunkSize = 2 Units gives 4 chunks
    assert len(chunks) == 4
    r = PL.state_aware_1f1b(chunks, groups, 2, 4)
    assert r["makespan"] == 46 and printed_as(r["bubble_ratio"], g["state_aware_chunk2_k2"])
    chunks4, groups4 = CK.build_chunks(lens, 4)    # section 5: ChunkSize = 4 Units gives 2 chunks
    assert len(chunks4) == 2
    r = PL.state_aware_1f1b(chunks4, groups4, 1, 4)
    assert r["bubble_ratio"] == Fraction(3, 5) and printed_as(r["bubble_ratio"], g["state_aware_chunk4_k1"])
    # the order of the input sequences does not matter to the chunked schedules
    for perm in ([1, 1, 2, 4], [2, 4, 1, 1]):
        c, gr = CK.build_chunks(perm, 2)
        assert PL.state_aware_1f1b(c, gr, 2, 4)["makespan"] == 46


def test_k1_figure_is_unreachable_in_the_stated_cost_model():
    """Section 4.3 prints 54.1 % for ChunkSize 2 Units, K = 1.  Every pass of that example lasts 2 or 4 Units, so any
    schedule's makespan is an even number of Units; work per stage is 24 Units, or 26 with the re-forward of
    the split sequence's first chunk.  No even makespan gives a ratio that prints as 54.1."""
    g = golden()
    target = g["state_aware_chunk2_k1"]
    for T in range(26, 400, 2):
        for work in (24, 26):
            assert not printed_as(Fraction(T - work, T), target), (T, work)
    chunks, groups = CK.build_chunks([4, 2, 1, 1], 2)
    r = PL.state_aware_1f1b(chunks, groups, 1, 4)
    assert r["busy"] == [26] * 4 and r["makespan"] % 2 == 0
    assert r["makespan"] == 62                      # what this reading gives: 58.06 %, recorded in the module header


@pytest.mark.parametrize("m,p", [(1, 1), (1, 4), (4, 4), (8, 4), (16, 8), (3, 5), (32, 2)])
def test_equal_microbatches_closed_form(m, p):
    """m equal micro-batches on p stages: bubble ratio (p-1)/(m+p-1), for both schedulers."""
    r = PL.one_f_one_b([3] * m, p)
    assert r["bubble_ratio"] == Fraction(p - 1, m + p - 1) and r["makespan"] == (m + p - 1) * 9
    chunks = [{"tokens": 3} for _ in range(m)]
    groups = [{"seq_id": -1, "chunks": [i]} for i in range(m)]
    assert PL.state_aware_1f1b(chunks, groups, 1, p)["makespan"] == r["makespan"]


def test_one_stage_has_no_bubble_and_work_is_conserved():
    rng = np.random.default_rng(5)
    for _ in range(60):
        lens = [int(x) for x in rng.integers(1, 40, size=int(rng.integers(1, 12)))]
        C = int(rng.integers(2, 30))
        K = int(rng.integers(1, 4))
        p = int(rng.integers(1, 6))
        chunks, groups = CK.build_chunks(lens, C)
        r = PL.state_aware_1f1b(chunks, groups, K, p, standalone_first=bool(rng.integers(0, 2)))
        st = CK.schedule_stats(chunks, groups, K)
        assert len(r["ops"]) == st["n_forward"] + st["n_backward"]
        refwd = sum(chunks[c]["tokens"] for g in groups for c in g["chunks"][:max(0, len(g["chunks"]) - K)])
        assert r["busy"] == [3 * sum(lens) + refwd] * p          # forward n + backward 2n (+ re-forwards)
        assert r["makespan"] >= r["busy"][0]
        if p == 1:
            assert r["bubble_ratio"] == 0
        s = PL.one_f_one_b(lens, p)
        assert s["busy"] == [3 * sum(lens)] * p and (p > 1 or s["bubble_ratio"] == 0)
        # lower bound: the first micro-batch must cross the pipeline forward and the last one backward
        assert s["makespan"] >= 3 * sum(lens) + (p - 1) * (lens[0] + 2 * lens[-1]) - (0 if p > 1 else 0) or p == 1


def test_more_kept_chunks_never_need_more_reforwards_and_k_ge_n_is_plain_1f1b():
    chunks, groups = CK.build_chunks([40, 3, 5, 8], 8)
    r1 = PL.state_aware_1f1b(chunks, groups, 1, 4)
    r5 = PL.state_aware_1f1b(chunks, groups, 5, 4)
    assert r1["busy"][0] - r5["busy"][0] == 4 * 8                 # K = 1 re-forwards the first four slices
    assert r5["busy"][0] == 3 * 56
