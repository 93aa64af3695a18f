"""Host planner of the library against the Python oracle: descriptors must be bit-exact (CPU only)."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import chunking as CK
from paper_2503_02356_amd import binding as B
from paper_2503_02356_amd import inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def assert_same_plan(lens, C, merge_tails=False):
    chunks, groups = CK.build_chunks(lens, C, merge_tails=merge_tails)
    p = B.cf_build_chunks_ex(lens, C, B.CF_PLAN_MERGE_TAILS) if merge_tails else B.cf_build_chunks(lens, C)
    assert p.n_chunks == len(chunks) and p.n_groups == len(groups)
    assert p.total_tokens == int(np.sum(lens)) and p.chunk_size == C
    assert p.n_segments == sum(len(c["segments"]) for c in chunks)
    for c, ch in enumerate(chunks):
        assert p.chunk_segments(c) == [tuple(s) for s in ch["segments"]]
        assert int(p.chunk_tokens[c]) == ch["tokens"] and int(p.chunk_prefix_len[c]) == ch["prefix_len"]
        assert int(p.chunk_group[c]) == ch["group"] and int(p.chunk_idx_in_group[c]) == ch["idx_in_group"]
        cu = np.concatenate([[0], np.cumsum([s[2] for s in ch["segments"]])])
        assert np.array_equal(p.chunk_cu_seqlens(c), cu)
    for g, gr in enumerate(groups):
        assert p.group(g) == gr["chunks"] and int(p.group_seq_id[g]) == gr["seq_id"]
    for K in (1, 2, 5):
        assert p.schedule(K) == CK.build_schedule(groups, K)
        assert p.schedule_stats(K) == CK.schedule_stats(chunks, groups, K)
    p.close()
    return len(chunks)


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "chunkflow.h")).read()
    declared = set(re.findall(r"\b(cf_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS), declared ^ set(B.EXPORTS)
    so = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(so, name), name
    assert B.cf_version() >= 100


def test_paper_examples():
    assert assert_same_plan([1, 1, 2, 4], 2) == 4
    assert assert_same_plan([1, 1, 2, 4], 4) == 2


def test_random_lists_bit_exact():
    rng = np.random.default_rng(11)
    for trial in range(1500):
        n = int(rng.integers(0, 40))
        C = int(rng.integers(1, 200))
        kind = trial % 3
        if kind == 0:
            lens = rng.integers(1, 3 * C + 2, size=n)
        elif kind == 1:
            lens = np.clip(np.rint(rng.lognormal(np.log(max(C / 8, 1)), 0.9, size=n)), 1, 5 * C).astype(np.int64)
        else:
            lens = rng.choice([1, C, C + 1, max(1, C // 2), 2 * C], size=n)     # boundary lengths, many ties
        assert_same_plan([int(x) for x in lens], C)


def test_merged_tails_bit_exact():
    assert assert_same_plan([5, 1, 1], 2, merge_tails=True) == 4
    assert assert_same_plan([5, 5], 4, merge_tails=True) == 4
    rng = np.random.default_rng(12)
    for trial in range(600):
        n = int(rng.integers(0, 40))
        C = int(rng.integers(1, 200))
        if trial % 2:
            lens = rng.integers(1, 4 * C + 2, size=n)
        else:
            lens = rng.choice([1, C, C + 1, max(1, C // 2), 2 * C, 2 * C + 1, 3 * C - 1], size=n)
        assert_same_plan([int(x) for x in lens], C, merge_tails=True)
    # flags = 0 is cf_build_chunks; unknown bits are refused
    a, b = B.cf_build_chunks_ex([9, 3, 3, 10, 1], 4, 0), B.cf_build_chunks([9, 3, 3, 10, 1], 4)
    assert [a.chunk_segments(c) for c in range(a.n_chunks)] == [b.chunk_segments(c) for c in range(b.n_chunks)]
    with pytest.raises(B.CfError):
        B.cf_build_chunks_ex([3], 2, 2)


@pytest.mark.parametrize("cfg,sd", [("tiny_fp32", 1), ("packed_8k", 1), ("long32k_mixed", 1),
                                    ("longtail_16k", 8), ("long256k_32k", 1)])
def test_workload_shapes(cfg, sd):
    count = lambda lens, C: len(CK.build_chunks(lens, C)[0])
    lens, C = inputs.seq_lens(cfg, 0, count, scale_down=sd)
    n = assert_same_plan([int(x) for x in lens], C)
    if cfg == "packed_8k":
        assert n == 16
    if cfg == "long32k_mixed":
        assert n == 12
    if cfg == "long256k_32k":
        assert n == 12


def test_errors():
    L = B.lib()
    out = ctypes.c_void_p(1234)
    one = np.array([3, 0], dtype=np.int64)
    ptr = one.ctypes.data_as(ctypes.c_void_p)
    assert L.cf_build_chunks(ptr, 2, 4, ctypes.byref(out)) == B.CF_EINVAL and out.value == 1234
    assert b"seq_lens[1]" in L.cf_last_error()
    assert L.cf_build_chunks(ptr, 1, 0, ctypes.byref(out)) == B.CF_EINVAL
    assert L.cf_build_chunks(ptr, 1, 2 ** 31, ctypes.byref(out)) == B.CF_EINVAL
    assert L.cf_build_chunks(ptr, -1, 4, ctypes.byref(out)) == B.CF_EINVAL
    assert L.cf_build_chunks(None, 1, 4, ctypes.byref(out)) == B.CF_EINVAL
    assert L.cf_build_chunks(ptr, 1, 4, None) == B.CF_EINVAL
    assert out.value == 1234
    L.cf_plan_free(None)
    p = B.cf_build_chunks([], 8)
    assert p.n_chunks == 0 and p.n_groups == 0 and p.schedule(1) == []
    with pytest.raises(B.CfError):
        B.cf_build_chunks([5, 9], 4).schedule(0)
    assert B.cf_count_pairs([0, 3, 5], [0, 3, 5]) == 6 + 3
    assert B.cf_count_pairs([0, 4], [0, 10]) == 4 * 6 + 10


def test_device_entry_points_reject_bad_arguments_without_a_gpu():
    """Argument checks happen on the host before any HIP call."""
    p = B.AttnFwdParams()
    assert B.lib().cf_attn_fwd(None, None) == B.CF_EINVAL
    p.dtype, p.head_dim, p.n_q_heads, p.n_kv_heads = B.CF_BF16, 96, 4, 2
    assert B.lib().cf_attn_fwd(ctypes.byref(p), None) == B.CF_EUNSUPPORTED
    p.head_dim, p.n_q_heads = 128, 5
    assert B.lib().cf_attn_fwd(ctypes.byref(p), None) == B.CF_EINVAL
    p.n_q_heads, p.n_tokens, p.n_kv_tokens, p.n_segments = 4, 16, 8, 1
    assert B.lib().cf_attn_fwd(ctypes.byref(p), None) == B.CF_EINVAL          # fewer keys than queries
    p.n_kv_tokens = 16
    assert B.lib().cf_attn_fwd(ctypes.byref(p), None) == B.CF_EINVAL          # NULL pointers
    assert b"NULL" in B.lib().cf_last_error()
    assert B.cf_attn_bwd_workspace_bytes(p) >= 4 * 16 * 4
    # a tile table needs a plausible record count, and a count needs a table (fake, aligned addresses: the
    # checks run on the host and nothing is dereferenced)
    for name in ("cu_seqlens_q", "cu_seqlens_k", "q", "k", "v", "o", "lse"):
        setattr(p, name, 0x1000)
    p.softmax_scale, p.q_stride_tok, p.q_stride_head, p.kv_stride_tok, p.kv_stride_head = 1.0, 512, 128, 256, 128
    p.o_stride_tok, p.o_stride_head = 512, 128
    p.q_tiles, p.n_q_tiles = 0x2000, 0
    assert B.lib().cf_attn_fwd(ctypes.byref(p), None) == B.CF_EINVAL and b"q_tiles" in B.lib().cf_last_error()
    p.q_tiles, p.n_q_tiles = 0, 1
    assert B.lib().cf_attn_fwd(ctypes.byref(p), None) == B.CF_EINVAL and b"q_tiles" in B.lib().cf_last_error()
    p.q_tiles, p.n_q_tiles = 0x2000, 3                                         # 16 tokens in 1 segment: exactly 1 tile
    assert B.lib().cf_attn_fwd(ctypes.byref(p), None) == B.CF_EINVAL and b"n_q_tiles" in B.lib().cf_last_error()
    b = B.AttnBwdParams()
    assert B.lib().cf_attn_bwd(None, None) == B.CF_EINVAL
    assert B.lib().cf_attn_bwd(ctypes.byref(b), None) < 0


@pytest.mark.parametrize("K", [1, 2, 3, 16])
def test_schedule_stats_match_oracle(K):
    rng = np.random.default_rng(11)
    for _ in range(20):
        lens = [int(x) for x in rng.integers(1, 400, size=rng.integers(1, 15))]
        C = int(rng.integers(8, 96))
        plan = B.cf_build_chunks(lens, C)
        chunks, groups = CK.build_chunks(lens, C)
        assert plan.schedule_stats(K) == CK.schedule_stats(chunks, groups, K)
        plan.close()


def test_schedule_stats_errors():
    plan = B.cf_build_chunks([5, 9], 4)
    with pytest.raises(B.CfError):
        plan.schedule_stats(0)
    assert B.lib().cf_schedule_stats(plan._h, 1, None) == -1
    plan.close()


def test_schedule_memory_is_bounded_by_k_times_chunk_size():
    """Section 4.2: kept activations never exceed K chunks; the paper's peak-memory table grows with ChunkSize."""
    from paper_2503_02356_amd.runner import schedule_memory
    lens = [40000, 700, 3000, 12000, 250, 90, 5000]
    prev = 0
    for C in (2048, 4096, 8192):
        plan = B.cf_build_chunks(lens, C)
        m = schedule_memory(plan, 1, 28, 4, 128)
        assert m["kept_activation_bytes"] == C * 28 * (2 * 128 * 2 + 4)
        assert m["state_bytes"] == 40000 * 4 * 128 * (4 + 8)
        assert m["kept_activation_bytes"] > prev
        prev = m["kept_activation_bytes"]
        m4 = schedule_memory(plan, 4, 28, 4, 128)
        assert m4["kept_activation_bytes"] <= 4 * m["kept_activation_bytes"] and m4["n_reforward"] < m["n_reforward"]
        plan.close()


def test_batch_entry_points_reject_bad_arguments_without_a_gpu():
    """Every chunk of a batch call is checked on the host before anything is enqueued."""
    L = B.lib()
    assert L.cf_attn_fwd_batch(None, 0, None) == B.CF_OK and L.cf_attn_bwd_batch(None, 0, None) == B.CF_OK
    assert L.cf_attn_fwd_batch(None, 2, None) == B.CF_EINVAL and L.cf_attn_bwd_batch(None, -1, None) == B.CF_EINVAL
    arr = (B.AttnFwdParams * 2)()
    for p in arr:
        p.dtype, p.head_dim, p.n_q_heads, p.n_kv_heads = B.CF_BF16, 128, 4, 2
        p.n_tokens, p.n_kv_tokens, p.n_segments = 16, 16, 1
    assert L.cf_attn_fwd_batch(arr, 2, None) == B.CF_EINVAL and b"NULL" in L.cf_last_error()
    arr[1].head_dim = 96
    assert L.cf_attn_fwd_batch(arr, 2, None) in (B.CF_EINVAL, B.CF_EUNSUPPORTED)


def test_q_tile_table_lists_every_tile_heaviest_first():
    """cf_attn_q_tiles against a direct enumeration: every 128-row tile of every segment exactly once, with its
    segment's bounds, ordered by the number of 64-key steps its last row needs (ties: segment, then tile)."""
    rng = np.random.default_rng(3)
    for trial in range(200):
        n = int(rng.integers(1, 12))
        lq = rng.integers(1, 700, size=n)
        prefix = rng.integers(0, 2, size=n) * rng.integers(0, 900, size=n)
        cu_q = np.concatenate([[0], np.cumsum(lq)])
        cu_k = np.concatenate([[0], np.cumsum(lq + prefix)])
        rows = []
        for g in range(n):
            for j in range(-(-int(lq[g]) // 128)):
                keys = min((j + 1) * 128, int(lq[g])) + int(prefix[g])
                rows.append((-(-(-keys // 64)) * -1, len(rows), int(cu_q[g]), int(lq[g]), int(cu_k[g]), int(lq[g] + prefix[g]), j, g))
        rows = sorted((-steps, i, *rest) for (steps, i, *rest) in rows)
        want = np.array([r[2:] + (0, 0) for r in rows], dtype=np.int32).reshape(-1, 8)
        got = B.cf_attn_q_tiles(cu_q, cu_k)
        assert np.array_equal(got, want), trial
    with pytest.raises(B.CfError):
        B.cf_attn_q_tiles([0, 4, 4], [0, 4, 4])             # empty segment
    with pytest.raises(B.CfError):
        B.cf_attn_q_tiles([0, 4], [0, 3])                   # fewer keys than queries


def test_missing_library_is_an_error_not_a_fallback(monkeypatch):
    """The binding has no other path than the built library: without it every call raises."""
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", os.path.join(ROOT, "no_such_dir", "libchunkflow.so"))
    with pytest.raises(RuntimeError, match="missing"):
        B.cf_build_chunks([3, 4], 4)
    with pytest.raises(RuntimeError, match="missing"):
        B.cf_attn_fwd(B.AttnFwdParams(), None)


def test_static_scratch_backward_refuses_oversized_chunks_on_the_host():
    """cf_attn_bwd_static decides on the host, before any HIP call, that a chunk's scratch (delta =
    n_q_heads * n_tokens * 4 bytes, plus the work list) does not fit its static buffer: CF_EINVAL on any machine.
    The pointers are never dereferenced on that path (fake, aligned, non-NULL addresses)."""
    fp = B.AttnFwdParams()
    fp.dtype, fp.flags, fp.n_q_heads, fp.n_kv_heads, fp.head_dim = B.CF_BF16, 0, 64, 8, 128
    fp.softmax_scale = 0.1
    fp.n_tokens, fp.n_kv_tokens, fp.n_segments = 70000, 70000, 1          # 64 * 70000 * 4 bytes > 16 MiB
    fake = 1 << 20
    for name in ("cu_seqlens_q", "cu_seqlens_k", "q", "k", "v", "o", "lse"):
        setattr(fp, name, fake)
    for name in ("q_stride_tok", "o_stride_tok"):
        setattr(fp, name, 64 * 128)
    fp.kv_stride_tok = 8 * 128
    fp.q_stride_head = fp.o_stride_head = fp.kv_stride_head = 128
    bp = B.AttnBwdParams()
    bp.f = fp
    bp.d_o = bp.d_q = bp.d_k = bp.d_v = fake
    bp.do_stride_tok = bp.dq_stride_tok = 64 * 128
    bp.dkv_stride_tok = 8 * 128
    bp.do_stride_head = bp.dq_stride_head = bp.dkv_stride_head = 128
    need = B.cf_attn_bwd_workspace_bytes(fp)
    assert need > B.CF_STATIC_SCRATCH_BYTES
    with pytest.raises(B.CfError) as e:
        B.cf_attn_bwd_static(bp, ctypes.c_void_p(0))
    assert e.value.code == B.CF_EINVAL and "static buffer" in str(e.value)
    hdr = open(os.path.join(ROOT, "include", "chunkflow.h")).read()
    assert re.search(r"#define\s+CF_STATIC_SCRATCH_BYTES\s+\(16\s*<<\s*20\)", hdr)


def test_pipeline_simulator_bit_exact_against_the_oracle():
    """cf_sim_1f1b / cf_sim_1f1b_sequences (sections 3.3, 4.3, 5) against oracle/pipeline.py in integer ticks:
    the paper's example and random batches, every K and stage count, both group orders."""
    from fractions import Fraction
    from oracle import pipeline as PL
    r = B.cf_sim_1f1b_sequences([4, 2, 1, 1], 4)
    assert (r["makespan"], r["busy_per_stage"]) == (56, 24) and Fraction(r["bubble_ticks"], r["total_ticks"]) == Fraction(4, 7)
    plan = B.cf_build_chunks([4, 2, 1, 1], 2)
    assert plan.sim_1f1b(2, 4)["makespan"] == 46 and plan.sim_1f1b(1, 4)["makespan"] == 62
    plan = B.cf_build_chunks([4, 2, 1, 1], 4)
    r = plan.sim_1f1b(1, 4)
    assert Fraction(r["bubble_ticks"], r["total_ticks"]) == Fraction(3, 5)
    rng = np.random.default_rng(17)
    for trial in range(400):
        n = int(rng.integers(1, 14))
        C = int(rng.integers(1, 40))
        lens = [int(x) for x in rng.integers(1, 4 * C + 2, size=n)]
        K, p = int(rng.integers(1, 5)), int(rng.integers(1, 7))
        merge = bool(trial % 5 == 0)
        chunks, groups = CK.build_chunks(lens, C, merge_tails=merge)
        plan = B.cf_build_chunks_ex(lens, C, B.CF_PLAN_MERGE_TAILS if merge else 0)
        for flags, first in ((0, True), (B.CF_SIM_PLAN_ORDER, False)):
            ref = PL.state_aware_1f1b(chunks, groups, K, p, standalone_first=first)
            got = plan.sim_1f1b(K, p, flags)
            assert got["makespan"] == ref["makespan"] and got["busy_per_stage"] == ref["busy"][0], (lens, C, K, p, flags)
            assert got["n_ops"] == len(ref["ops"]) and got["total_ticks"] == p * ref["makespan"]
            assert Fraction(got["bubble_ticks"], got["total_ticks"]) == ref["bubble_ratio"]
        ref = PL.one_f_one_b(lens, p)
        got = B.cf_sim_1f1b_sequences(lens, p)
        assert got["makespan"] == ref["makespan"] and got["busy_per_stage"] == ref["busy"][0]
        plan.close()


def test_pipeline_simulator_errors():
    plan = B.cf_build_chunks([5, 3], 4)
    for K, p, flags in ((0, 4, 0), (1, 0, 0), (1, 4, 8)):
        with pytest.raises(B.CfError) as e:
            plan.sim_1f1b(K, p, flags)
        assert e.value.code == B.CF_EINVAL
    with pytest.raises(B.CfError):
        B.cf_sim_1f1b_sequences([3, 0], 2)
    assert B.cf_sim_1f1b_sequences([], 3)["makespan"] == 0
