"""Pins for the chunk-construction and scheduling oracle (CPU only).

The paper fixes: the chunk counts of its worked example (tests/golden/paper_examples.txt), that long
sequences are cut into ChunkSize slices and short ones bin-packed into as few bins as the packing
attempt manages (Algorithm 1), the forward/backward order inside a dependency group and the number
of repeated forward passes (section 4.2).  The particular packing heuristic is the oracle's own
reading; it is checked here for validity and against exhaustive search, not against the paper.
"""
import itertools
import os

import numpy as np
import pytest

from oracle import chunking as CK

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_examples.txt")


def golden_cases():
    out = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        c, lens, n = [x.strip() for x in line.split(";")]
        out.append((int(c), [int(x) for x in lens.split()], int(n)))
    return out


@pytest.mark.parametrize("C,lens,n_chunks", golden_cases())
def test_paper_worked_example(C, lens, n_chunks):
    chunks, groups = CK.build_chunks(lens, C)
    assert len(chunks) == n_chunks


def test_paper_example_structure():
    # ChunkSize 2: the 4-Unit sequence gives two dependent slices; the 2-Unit sequence is one full
    # standalone chunk; the two 1-Unit sequences share one exactly-full chunk.
    chunks, groups = CK.build_chunks([1, 1, 2, 4], 2)
    assert [c["segments"] for c in chunks] == [[(3, 0, 2)], [(3, 2, 2)], [(2, 0, 2)], [(0, 0, 1), (1, 0, 1)]]
    assert [c["prefix_len"] for c in chunks] == [0, 2, 0, 0]
    assert [g["seq_id"] for g in groups] == [3, -1, -1] and groups[0]["chunks"] == [0, 1]
    chunks, _ = CK.build_chunks([1, 1, 2, 4], 4)
    assert [c["segments"] for c in chunks] == [[(3, 0, 4)], [(0, 0, 1), (1, 0, 1), (2, 0, 2)]]


def check_valid(lens, C, chunks, groups):
    seen = {i: np.zeros(L, int) for i, L in enumerate(lens)}
    for cid, c in enumerate(chunks):
        assert 1 <= c["tokens"] <= C and c["tokens"] == sum(s[2] for s in c["segments"])
        for (sid, st, n) in c["segments"]:
            seen[sid][st:st + n] += 1
        g = groups[c["group"]]
        assert g["chunks"][c["idx_in_group"]] == cid
        if g["seq_id"] >= 0:                       # dependent slice
            assert len(c["segments"]) == 1 and lens[g["seq_id"]] > C
            sid, st, n = c["segments"][0]
            assert sid == g["seq_id"] and st == c["prefix_len"] == c["idx_in_group"] * C
            last = c["idx_in_group"] == len(g["chunks"]) - 1
            assert n == C or (last and n == lens[sid] - st)
        else:
            assert c["prefix_len"] == 0 and len(g["chunks"]) == 1
            assert all(st == 0 and n == lens[sid] and n <= C for (sid, st, n) in c["segments"])
            assert [s[0] for s in c["segments"]] == sorted(s[0] for s in c["segments"])
    assert all((v == 1).all() for v in seen.values())       # every token exactly once


def optimal_bins(items, C):
    """Exhaustive minimum number of bins (tiny inputs only)."""
    n = len(items)
    for b in range(1, n + 1):
        for assign in itertools.product(range(b), repeat=n):
            load = [0] * b
            for x, a in zip(items, assign):
                load[a] += x
            if max(load) <= C:
                return b
    return n


def test_random_lists_are_valid_and_near_optimal():
    rng = np.random.default_rng(0)
    for trial in range(300):
        n = int(rng.integers(0, 9))
        C = int(rng.integers(1, 40))
        lens = [int(x) for x in rng.integers(1, 3 * C + 2, size=n)]
        chunks, groups = CK.build_chunks(lens, C)
        check_valid(lens, C, chunks, groups)
        short = [x for x in lens if x <= C]
        packed = sum(1 for g in groups if g["seq_id"] < 0)
        assert packed >= -(-sum(short) // C)
        if len(short) <= 7:
            assert packed >= optimal_bins(short, C)           # optimum is a lower bound
            assert packed <= optimal_bins(short, C) + 2       # and the heuristic stays close
        n_long = sum(-(-x // C) for x in lens if x > C)
        assert len(chunks) == n_long + packed


def test_bad_arguments():
    for lens, C in (([3, 0], 4), ([3], 0), ([-1], 4)):
        with pytest.raises(ValueError):
            CK.build_chunks(lens, C)
    assert CK.build_chunks([], 8) == ([], [])


@pytest.mark.parametrize("N,K", [(1, 1), (4, 1), (4, 2), (4, 4), (3, 7), (7, 3)])
def test_schedule_counts_and_order(N, K):
    ids = list(range(10, 10 + N))
    ops = CK.schedule_group(ids, K)
    n_fwd = sum(1 for op, _ in ops if op != CK.BWD)
    n_bwd = sum(1 for op, _ in ops if op == CK.BWD)
    # section 4.2: the first N-K chunks run forward twice when N > K
    assert n_fwd == (N + (N - K) if N > K else N) and n_bwd == N
    live, first_fwd_done, bwd_done = set(), set(), set()
    for op, c in ops:
        m = c - 10
        if op in (CK.FWD_KEEP, CK.FWD_DISCARD):
            assert all(x in first_fwd_done for x in range(m))        # ascending forward dependency
            first_fwd_done.add(m)
            if op == CK.FWD_KEEP:
                live.add(m)
                assert len(live) <= K                                 # at most K chunks' activations
        else:
            assert m in live                                          # backward needs kept activations
            assert all(x in bwd_done for x in range(m + 1, N))        # descending backward dependency
            live.discard(m)
            bwd_done.add(m)
    assert bwd_done == set(range(N)) and not live


def test_schedule_whole_plan_groups_contiguous():
    chunks, groups = CK.build_chunks([9, 2, 30, 3], 8)
    ops = CK.build_schedule(groups, 1)
    seen_groups = [chunks[c]["group"] for _, c in ops]
    assert seen_groups == sorted(seen_groups)
    with pytest.raises(ValueError):
        CK.build_schedule(groups, 0)


# ---- schedule_stats: what section 4.2 says a schedule costs and keeps --------------------------------

@pytest.mark.parametrize("N,K", [(1, 1), (4, 1), (4, 2), (4, 4), (4, 9), (8, 3)])
def test_schedule_stats_single_long_sequence(N, K):
    """One sequence of N full chunks (closed forms from section 4.2: the first N-K chunks run forward
    twice; at most K chunks' activations are kept; the key/value state covers the whole sequence)."""
    C = 16
    chunks, groups = CK.build_chunks([N * C], C) if N > 1 else CK.build_chunks([C], C)
    st = CK.schedule_stats(chunks, groups, K)
    assert st["n_backward"] == N
    assert st["n_reforward"] == max(0, N - K) and st["n_forward"] == N + max(0, N - K)
    assert st["peak_kept_chunks"] == min(N, K) and st["peak_kept_tokens"] == min(N, K) * C
    assert st["state_tokens"] == (N * C if N > 1 else 0)


def test_schedule_stats_k1_keeps_one_chunk_at_a_time():
    """Section 4.2 for K = 1: at any time at most one chunk's activations are stored, whatever the batch."""
    rng = np.random.default_rng(5)
    for _ in range(30):
        lens = [int(x) for x in rng.integers(1, 200, size=rng.integers(1, 12))]
        C = int(rng.integers(8, 64))
        chunks, groups = CK.build_chunks(lens, C)
        st = CK.schedule_stats(chunks, groups, 1)
        assert st["peak_kept_chunks"] == 1 and st["peak_kept_tokens"] <= C
        long_chunks = sum(len(g["chunks"]) - 1 for g in groups if g["seq_id"] >= 0)
        assert st["n_reforward"] == long_chunks          # every chunk but the last of each split sequence


def test_schedule_stats_kept_memory_follows_chunk_size():
    """The trend of the paper's peak-memory table: with K fixed, a larger ChunkSize keeps more tokens
    (the bound K * ChunkSize is reached as soon as a sequence is split), and K * ChunkSize bounds it."""
    lens = [40000, 700, 3000, 12000, 250, 90, 5000]
    peaks = []
    for C in (2048, 4096, 8192):
        chunks, groups = CK.build_chunks(lens, C)
        for K in (1, 2, 4):
            st = CK.schedule_stats(chunks, groups, K)
            assert st["peak_kept_tokens"] <= K * C
            assert st["state_tokens"] == 40000
        peaks.append(CK.schedule_stats(chunks, groups, 1)["peak_kept_tokens"])
    assert peaks == [2048, 4096, 8192]


# ---------------------------------------------------------------- merged tails (variant of Algorithm 1)

def check_valid_merged(lens, C, chunks, groups):
    """What must hold for any reading of 'the last slice joins the bin-packing': every token once, chunks within
    ChunkSize, full slices first in their group, at most one tail per chunk and that chunk last in the tail's group."""
    seen = {i: np.zeros(L, int) for i, L in enumerate(lens)}
    for cid, c in enumerate(chunks):
        assert 1 <= c["tokens"] <= C and c["tokens"] == sum(s[2] for s in c["segments"])
        for (sid, st, n) in c["segments"]:
            seen[sid][st:st + n] += 1
        g = groups[c["group"]]
        assert g["chunks"][c["idx_in_group"]] == cid
        assert [s[0] for s in c["segments"]] == sorted(s[0] for s in c["segments"])
        slices = [(sid, st, n) for (sid, st, n) in c["segments"] if lens[sid] > C]
        assert len(slices) <= 1
        if g["seq_id"] >= 0:
            (sid, st, n), = slices
            assert sid == g["seq_id"] and st == c["prefix_len"] == c["idx_in_group"] * C
            if n == C:
                assert len(c["segments"]) == 1                       # a full slice is alone
            else:
                assert c["idx_in_group"] == len(g["chunks"]) - 1 and n == lens[sid] - st
        else:
            assert not slices and c["prefix_len"] == 0 and len(g["chunks"]) == 1
        assert all(st == 0 and n == lens[sid] for (sid, st, n) in c["segments"] if lens[sid] <= C)
    assert all((v == 1).all() for v in seen.values())


def test_merged_tails_worked_examples():
    # 5 tokens, ChunkSize 2: two full slices and a 1-token tail (prefix 4).  Items of length 1: the tail (sequence 0),
    # sequences 1 and 2; 3 tokens need 2 bins; tail -> bin 0, sequence 1 -> bin 1, sequence 2 -> bin 0 (tie: lowest).
    chunks, groups = CK.build_chunks([5, 1, 1], 2, merge_tails=True)
    assert [c["segments"] for c in chunks] == [[(0, 0, 2)], [(0, 2, 2)], [(0, 4, 1), (2, 0, 1)], [(1, 0, 1)]]
    assert [c["prefix_len"] for c in chunks] == [0, 2, 4, 0]
    assert groups == [{"seq_id": 0, "chunks": [0, 1, 2]}, {"seq_id": -1, "chunks": [3]}]
    # without the option the tail is a chunk of its own and the two short sequences share one
    plain, _ = CK.build_chunks([5, 1, 1], 2)
    assert [c["segments"] for c in plain] == [[(0, 0, 2)], [(0, 2, 2)], [(0, 4, 1)], [(1, 0, 1), (2, 0, 1)]]
    # two tails never share a chunk, even when they would fit: 2 bins although 2 tokens fit one
    chunks, groups = CK.build_chunks([5, 5], 4, merge_tails=True)
    assert [c["segments"] for c in chunks] == [[(0, 0, 4)], [(1, 0, 4)], [(0, 4, 1)], [(1, 4, 1)]]
    assert [g["chunks"] for g in groups] == [[0, 2], [1, 3]]
    # a sequence that is a whole number of chunks has no tail; nothing changes
    assert CK.build_chunks([1, 1, 2, 4], 2, merge_tails=True) == CK.build_chunks([1, 1, 2, 4], 2)


def test_merged_tails_random_lists_are_valid_and_save_chunks():
    rng = np.random.default_rng(5)
    fewer = 0
    for trial in range(400):
        n = int(rng.integers(0, 10))
        C = int(rng.integers(1, 40))
        lens = [int(x) for x in rng.integers(1, 4 * C + 2, size=n)]
        chunks, groups = CK.build_chunks(lens, C, merge_tails=True)
        check_valid_merged(lens, C, chunks, groups)
        plain, _ = CK.build_chunks(lens, C)
        assert len(chunks) >= -(-sum(lens) // C)            # cannot beat the token bound
        fewer += len(chunks) < len(plain)
        # schedules stay well-formed: every chunk forward and backward, groups contiguous
        ops = CK.build_schedule(groups, 2)
        assert sorted(c for op, c in ops if op == CK.BWD) == list(range(len(chunks)))
        st = CK.schedule_stats(chunks, groups, 2)
        assert st["state_tokens"] == max([x for x in lens if x > C], default=0)
    assert fewer > 50                                       # the point of the variant
