"""Algorithm 2 with a bounded activation pool (paper section 4.2): the executor that really discards.  Parity with
the oracle for several K, the failure modes that show the discard is real, and the measured memory trend."""
import numpy as np
import pytest
import torch

from paper_2503_02356_amd import binding as B
from paper_2503_02356_amd import inputs
from paper_2503_02356_amd.executor import SlotExecutor
from paper_2503_02356_amd.runner import schedule_memory
from tests import parity as P

pytestmark = pytest.mark.gpu
LENS, C, HQ, HKV, D = [900, 40, 300, 1500, 77, 256], 256, 4, 2, 128


def make(K, seed=31, lens=LENS, chunk=C, dtype="bf16", D_=D):
    plan = B.cf_build_chunks(lens, chunk)
    vals = lambda sid, L: inputs.seq_values(seed, sid, lens[sid], HQ, HKV, D_, dtype)
    return plan, SlotExecutor(plan, HQ, HKV, D_, dtype, K).load(vals)


@pytest.mark.parametrize("K,dtype,D_", [(1, "bf16", 128), (2, "bf16", 128), (3, "bf16", 128), (8, "bf16", 128), (1, "fp32", 64)])
def test_executor_matches_the_oracle_for_every_k(K, dtype, D_):
    plan, ex = make(K, dtype=dtype, D_=D_)
    ex.run()
    ref = P.run_oracle(LENS, HQ, HKV, D_, dtype, seed=31)
    print(K, dtype, P.check(ex.results(), ref, dtype, f"executor K={K}"))
    st = plan.schedule_stats(K)
    assert ex.n_forward == st["n_forward"] and ex.n_backward == st["n_backward"]
    assert ex.peak_slots == st["peak_kept_chunks"] <= K
    # everything the pool held was given back and poisoned
    for s in ex.slots + [ex.scratch]:
        assert s.chunk is None and torch.isnan(s.o).all() and torch.isnan(s.lse).all()


def test_backward_of_a_discarded_chunk_needs_its_second_forward():
    """Remove the re-forward that Algorithm 2 schedules for a discarded chunk: its backward finds no activations
    (the first forward's went to the scratch slot, which was poisoned) and the executor refuses to go on."""
    plan, ex = make(1)
    ops = plan.schedule(1)
    discarded = {c for op, c in ops if op == B.CF_OP_FWD_DISCARD}
    assert discarded
    seen, cut = set(), []
    for op, c in ops:
        if op == B.CF_OP_FWD_KEEP and c in discarded and c not in seen:
            seen.add(c)
            continue                                   # drop the second forward
        cut.append((op, c))
    with pytest.raises(RuntimeError, match="without kept activations"):
        ex.run(cut)


def test_forward_passes_of_a_group_out_of_order_are_refused():
    """Section 4.2: chunks of one sequence run forward in ascending order (a chunk's keys enter the state at its
    first forward).  Swapping two forwards of a split sequence is caught."""
    plan, ex = make(8)
    ops = plan.schedule(8)
    g = [x for x in range(plan.n_groups) if int(plan.group_seq_id[x]) >= 0][0]
    first, second = plan.group(g)[0], plan.group(g)[1]
    i, j = ops.index((B.CF_OP_FWD_KEEP, first)), ops.index((B.CF_OP_FWD_KEEP, second))
    ops[i], ops[j] = ops[j], ops[i]
    with pytest.raises(RuntimeError, match="ascending order"):
        ex.run(ops)


def test_pool_of_k_slots_cannot_hold_more_than_k_chunks():
    plan, ex = make(1)
    with pytest.raises(RuntimeError, match="more than K kept chunks"):
        ex.run(plan.schedule(2))                       # a K = 2 schedule on a pool of one slot


def test_measured_memory_follows_k_times_chunk_size():
    """Peak device memory of a run, measured by the allocator, against the executor's own account and against
    cf_schedule_stats' prediction: going from K = 1 to K = 3 costs exactly two more chunk-sized slots."""
    lens, chunk = [6000, 300, 500], 1024
    peaks = {}
    for K in (1, 3):
        plan = B.cf_build_chunks(lens, chunk)
        vals = lambda sid, L: inputs.seq_values(5, sid, lens[sid], HQ, HKV, D, "bf16")
        ex = SlotExecutor(plan, HQ, HKV, D, "bf16", K).load(vals)
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        torch.cuda.reset_peak_memory_stats()
        base = torch.cuda.memory_allocated()
        ex.run()
        peaks[K] = torch.cuda.max_memory_allocated() - base
        account = sum(ex.device_bytes().values())
        pred = schedule_memory(plan, K, HQ, HKV, D)
        print(K, "measured", peaks[K], "accounted", account, "kept-activation bound", pred["kept_activation_bytes"],
              "state", pred["state_bytes"], flush=True)
        assert account <= peaks[K] <= account * 1.05 + (4 << 20)        # descriptors and allocator rounding on top
        assert pred["kept_activation_bytes"] <= ex.device_bytes()["activation_slots"]
        assert pred["state_bytes"] == ex.device_bytes()["state"]
        del ex
    slot = chunk * HQ * (2 * D * 2 + 4)
    assert abs((peaks[3] - peaks[1]) - 2 * slot) <= (2 << 20)
