"""ORACLE -- test infrastructure only: pipeline bubble ratios of 1F1B schedules in plain Python.

Follows the paper's cost model for its pipeline examples (section 3.3): the time of a micro-batch is
proportional to its length, a backward pass takes twice as long as the forward pass, and
    bubble ratio = total bubble time / total execution time            (equation 1)
summed over the pipeline stages.  Times are integer ticks (forward of n tokens = n ticks, backward 2n).

one_f_one_b       the standard 1F1B schedule over micro-batches of given lengths (section 3.3)
state_aware_1f1b  1F1B over the chunks of a plan in the order Algorithm 2 gives them (section 4.3)

Pins (tests/test_oracle_pipeline.py): the ratios the paper prints for its four-sequence example with four
stages -- 57.14 % (standard 1F1B, lengths 4, 2, 1, 1 Units), 42.8 % (four equal sequences), 60 % (ChunkSize
4 Units) and 47.8 % (ChunkSize 2 Units, K = 2) -- plus the closed form (p-1)/(m+p-1) for m equal
micro-batches and conservation checks.  The paper's fifth figure, 54.1 % for ChunkSize 2 Units with K = 1, is
NOT reachable in this cost model by ANY schedule: every pass there lasts an even number of Units (chunks of
2 Units: 2 forward, 4 backward), so the makespan T is even, and neither (T-26)/T (re-forward counted as work)
nor (T-24)/T (counted as bubble) rounds or truncates to 54.1 % for an even T (the test enumerates them).
PARITY UNPINNED for that one figure; the schedule below gives 58.06 % there.

Readings (the paper draws these schedules in figures that are not available):
  * the standard schedule is Megatron-LM's: stage s (0-based, p stages) runs p-1-s warm-up forwards, then
    alternates one forward and one backward, then drains; micro-batches in the given order;
  * state-aware 1F1B keeps that shape but takes its forward-type passes (first forwards and the re-forwards
    of discarded chunks) and its backward passes from Algorithm 2's op list, each kind in list order, and a
    pass may only run on a stage once the previous op of the SAME dependency group in Algorithm 2's list has
    run there (a re-forward follows the backward of the later chunk; a backward follows its kept forward).
    A stage starts a forward that keeps activations while it holds fewer than p-s kept chunks, or when
    the next backward is not yet allowed (that is how K = 2 lets the last stage hold two chunks); otherwise
    it runs the next backward.  A discarded forward holds nothing;
  * standalone chunks are scheduled before the dependent groups (the numbering of the paper's chunk
    figure: "Chunk 1 to Chunk 3" standalone, "Chunk 4 to Chunk 7" dependent); with the other order the
    K = 2 example gives 45.45 % instead of the printed 47.8 %.
"""
from fractions import Fraction

from . import chunking as CK


def _timeline(stage_orders, is_backward, ticks):
    """Start every op of every stage as early as its stage and its pipeline neighbour allow.

    stage_orders[s]: op ids in the order stage s runs them.  A forward-type op waits for the same op on
    stage s-1, a backward op for the same op on stage s+1.  Returns (makespan, busy ticks per stage).
    """
    p = len(stage_orders)
    end = [dict() for _ in range(p)]
    pos, free, busy = [0] * p, [0] * p, [0] * p
    remaining = sum(len(o) for o in stage_orders)
    while remaining:
        moved = False
        for s in range(p):
            while pos[s] < len(stage_orders[s]):
                op = stage_orders[s][pos[s]]
                if is_backward[op]:
                    ready = 0 if s == p - 1 else end[s + 1].get(op)
                else:
                    ready = 0 if s == 0 else end[s - 1].get(op)
                if ready is None:
                    break
                start = max(free[s], ready)
                end[s][op] = free[s] = start + ticks[op]
                busy[s] += ticks[op]
                pos[s] += 1
                remaining -= 1
                moved = True
        if not moved:
            raise RuntimeError("the stage orders deadlock")
    return max(free), busy


def _result(makespan, busy):
    p = len(busy)
    return {"makespan": makespan, "busy": busy, "n_stages": p,
            "bubble_ratio": Fraction(p * makespan - sum(busy), p * makespan) if makespan else Fraction(0)}


def one_f_one_b(lengths, n_stages):
    """Standard 1F1B (section 3.3) over micro-batches of the given lengths, in the given order."""
    m, p = len(lengths), int(n_stages)
    if p < 1 or any(int(x) < 1 for x in lengths):
        raise ValueError("n_stages and every length must be >= 1")
    # op ids: forward of micro-batch i = i, backward = m + i
    orders = []
    for s in range(p):
        warm = min(p - 1 - s, m)
        seq = list(range(warm))
        for i in range(m - warm):
            seq += [warm + i, m + i]
        seq += [m + i for i in range(m - warm, m)]
        orders.append(seq)
    ticks = [int(x) for x in lengths] + [2 * int(x) for x in lengths]
    return _result(*_timeline(orders, [False] * m + [True] * m, ticks))


def _stage_order(ops, prev_in_group, limit):
    """1F1B with prerequisites on one stage: the order of Algorithm 2's ops there (indices into ops)."""
    fwd = [i for i, (op, _) in enumerate(ops) if op != CK.BWD]
    bwd = [i for i, (op, _) in enumerate(ops) if op == CK.BWD]
    ran, order = set(), []
    fi = bi = held = 0
    allowed = lambda i: prev_in_group[i] is None or prev_in_group[i] in ran
    while fi < len(fwd) or bi < len(bwd):
        f_ok = fi < len(fwd) and allowed(fwd[fi])
        b_ok = bi < len(bwd) and allowed(bwd[bi])
        keeps = f_ok and ops[fwd[fi]][0] == CK.FWD_KEEP
        if f_ok and (not keeps or held < limit or not b_ok):
            i = fwd[fi]
            fi += 1
            held += 1 if keeps else 0
        elif b_ok:
            i = bwd[bi]
            bi += 1
            held -= 1
        else:
            raise RuntimeError("Algorithm 2's order cannot be followed")
        ran.add(i)
        order.append(i)
    return order


def state_aware_1f1b(chunks, groups, K, n_stages, standalone_first=True):
    """State-aware 1F1B (section 4.3) over the chunks of a plan (oracle.chunking.build_chunks)."""
    p = int(n_stages)
    if p < 1:
        raise ValueError("n_stages must be >= 1")
    groups = list(groups)
    if standalone_first:        # stable: standalone chunks keep their order, then the dependent groups in theirs
        groups = [g for g in groups if g["seq_id"] < 0] + [g for g in groups if g["seq_id"] >= 0]
    ops = CK.build_schedule(groups, K)
    group_of = {c: n for n, g in enumerate(groups) for c in g["chunks"]}
    prev_in_group, last = [], {}
    for i, (_, c) in enumerate(ops):
        prev_in_group.append(last.get(group_of[c]))
        last[group_of[c]] = i
    orders = [_stage_order(ops, prev_in_group, p - s) for s in range(p)]
    is_backward = [op == CK.BWD for op, _ in ops]
    ticks = [chunks[c]["tokens"] * (2 if op == CK.BWD else 1) for op, c in ops]
    out = _result(*_timeline(orders, is_backward, ticks))
    out["ops"] = ops
    return out
