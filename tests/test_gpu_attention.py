"""GPU parity: the library's chunked attention against the fp64 oracle's UNSPLIT attention, element by
element, re-indexed through the plan.  Tolerances are the north-star's (tests/parity.py)."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import attention as OA
from paper_2503_02356_amd import binding as B
from paper_2503_02356_amd import inputs
from paper_2503_02356_amd.runner import ChunkAttention
from tests import parity as P

pytestmark = pytest.mark.gpu
SCALAR = B.CF_FLAG_SCALAR_KERNELS


def test_config1_tiny_fp32_full():
    lens, C = inputs.seq_lens("tiny_fp32", 0, P.oracle_count_chunks)
    lens = [int(x) for x in lens]
    got, eng = P.run_gpu(lens, C, 1, 1, 64, "fp32", seed=1)
    assert [ch["P"] for ch in eng.chunks[:3]] == [0, 256, 512]
    ref = P.run_oracle(lens, 1, 1, 64, "fp32", seed=1)
    errs = P.check(got, ref, "fp32", "config 1")
    print("config1", errs)


@pytest.mark.parametrize("dtype,D,flags", [("fp32", 128, 0), ("bf16", 64, 0), ("bf16", 128, SCALAR), ("bf16", 128, 0)])
def test_small_mixed_plan(dtype, D, flags):
    """Long sequence split in 4 (non-dividing tail) + packed short ones, GQA 6/2, ragged lengths."""
    lens = [700, 33, 1, 120, 64, 65, 17, 128, 5, 250]
    C = 200
    got, _ = P.run_gpu(lens, C, 6, 2, D, dtype, seed=2, flags=flags)
    ref = P.run_oracle(lens, 6, 2, D, dtype, seed=2)
    print(dtype, D, flags, P.check(got, ref, dtype, f"{dtype} D={D} flags={flags}"))


@pytest.mark.parametrize("cfg,sd,Hq,Hkv", [("packed_8k", 16, 28, 4), ("long32k_mixed", 16, 28, 4),
                                           ("longtail_16k", 64, 32, 8), ("long256k_32k", 64, 16, 2)])
def test_scaled_down_configs_bf16(cfg, sd, Hq, Hkv):
    """Structurally identical small instances of configs 2-5 (chunk size and lengths divided by sd)."""
    lens, C = inputs.seq_lens(cfg, 0, P.oracle_count_chunks, scale_down=sd)
    lens = [int(x) for x in lens]
    if cfg == "longtail_16k":
        lens = lens[:120] + [max(lens)]          # keep the oracle's work to seconds; keep one long sequence
    got, eng = P.run_gpu(lens, C, Hq, Hkv, 128, "bf16", seed=3)
    ref = P.run_oracle(lens, Hq, Hkv, 128, "bf16", seed=3)
    print(cfg, "chunks", len(eng.chunks), P.check(got, ref, "bf16", cfg))


@pytest.mark.parametrize("flags", [SCALAR, 0])
def test_edge_cases(flags):
    cases = [
        ([1], 8),                          # one token
        ([1, 1, 1, 1, 1, 1, 1, 1], 8),     # eight one-token documents in one chunk
        ([129], 128),                      # tail slice of one token with a 128-token prefix
        ([127, 128, 129, 2], 128),         # around a tile edge
        ([513], 64),                       # nine slices, last has one token
        ([64] * 9, 192),
    ]
    for lens, C in cases:
        got, _ = P.run_gpu(lens, C, 4, 2, 128, "bf16", seed=4, flags=flags)
        ref = P.run_oracle(lens, 4, 2, 128, "bf16", seed=4)
        P.check(got, ref, "bf16", f"lens={lens} C={C}")


@pytest.mark.parametrize("flags", [SCALAR, 0])
def test_many_tiny_documents_in_one_chunk(flags):
    """More than 64 documents in one chunk (the on-device tile search walks the segment list in groups of 64,
    the dK/dV work list has one item per document) and more than 128: 300 documents of 1..40 tokens."""
    rng = np.random.default_rng(12)
    lens = [int(x) for x in rng.integers(1, 41, size=300)]
    C = sum(lens[:150]) + 7                     # two or three packed chunks, each with far more than 64 documents
    got, eng = P.run_gpu(lens, C, 4, 2, 128, "bf16", seed=6, flags=flags)
    assert max(len(ch["segs"]) for ch in eng.chunks) > 128
    ref = P.run_oracle(lens, 4, 2, 128, "bf16", seed=6)
    P.check(got, ref, "bf16", "300 tiny documents")


@pytest.mark.parametrize("dtype,D,flags,K,fused", [("bf16", 128, 0, None, False), ("bf16", 128, 0, 1, False),
                                                    ("bf16", 128, 0, None, True), ("bf16", 128, SCALAR, None, False),
                                                    ("fp32", 64, 0, 2, False)])
def test_merged_tails_plan(dtype, D, flags, K, fused):
    """Algorithm 1's variant that packs the last slice of a split sequence with short sequences: chunks whose
    segments mix a slice that reads its sequence's key/value state with whole short sequences."""
    lens = [700, 40, 300, 33, 1000, 129, 64, 5, 450, 17, 260, 90]
    C = 256
    got, eng = P.run_gpu(lens, C, 4, 2, D, dtype, seed=9, flags=flags, K=K, fused_launch=fused, merge_tails=True)
    assert sum(ch["merged"] for ch in eng.chunks) >= 2           # 700 -> tail 188, 1000 -> tail 232, 450 -> tail 194
    ref = P.run_oracle(lens, 4, 2, D, dtype, seed=9)
    P.check(got, ref, dtype, f"merged tails {dtype} D={D} flags={flags} K={K} fused={fused}")


@pytest.mark.parametrize("merge_tails", [False, True])
def test_tile_table_and_on_device_search_give_the_same_result(merge_tails):
    """With the host-built tile table (the runner's default) and without it (the kernels search cu_seqlens) the
    forward and dQ kernels do the same work in a different order: O, LSE and dQ must be bitwise equal, and both
    must match the oracle."""
    lens = [700, 40, 300, 33, 1000, 129, 64, 5, 450, 17, 260, 90, 128, 256]
    a, _ = P.run_gpu(lens, 256, 4, 2, 128, "bf16", seed=13, merge_tails=merge_tails, tile_tables=True)
    b, _ = P.run_gpu(lens, 256, 4, 2, 128, "bf16", seed=13, merge_tails=merge_tails, tile_tables=False)
    for sid in a:
        for name in ("o", "lse", "dq"):
            assert np.array_equal(a[sid][name], b[sid][name]), (sid, name)
    ref = P.run_oracle(lens, 4, 2, 128, "bf16", seed=13)
    P.check(a, ref, "bf16", "with tile tables")
    P.check(b, ref, "bf16", "without tile tables")


@pytest.mark.parametrize("K", [None, 1])
def test_step_captured_in_a_hip_graph_replays_correctly(K):
    """A whole step recorded into a HIP graph: every replay, with eager work of the same engine and
    synchronisations in between, must reproduce the eager results (forward and dQ bitwise; dK/dV, summed by
    atomics, within the tolerance against the oracle)."""
    lens = [700, 40, 300, 33, 1000, 129, 64, 5, 450]
    plan = B.cf_build_chunks(lens, 256)
    vals = lambda sid, L: inputs.seq_values(21, sid, lens[sid], 4, 2, 128, "bf16")
    eng = ChunkAttention(plan, 4, 2, 128, "bf16").load(vals)
    eng.zero_grads()
    if K is None:
        eng.run_forward(); eng.run_backward()
    else:
        eng.run_schedule(K)
    eager = eng.results()
    ref = P.run_oracle(lens, 4, 2, 128, "bf16", seed=21)
    P.check(eager, ref, "bf16", "eager")
    graph = eng.capture_step(K)
    for replay in range(3):
        for ch in eng.chunks:                      # eager work between the replays: spoil the outputs
            ch["o"].fill_(7.0); ch["d_q"].fill_(7.0); ch["lse"].fill_(7.0)
        eng.grad_arena.fill_(3.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = eng.results()
        for sid in got:
            for name in ("o", "lse", "dq"):
                assert np.array_equal(got[sid][name], eager[sid][name]), (replay, sid, name)
        P.check(got, ref, "bf16", f"graph replay {replay}")


def test_recompute_schedule_gives_same_result():
    """Algorithm 2 with K=1: the first N-1 chunks run forward twice; results must not change."""
    lens = [900, 40, 300]
    a, _ = P.run_gpu(lens, 256, 4, 2, 128, "bf16", seed=5)
    b, _ = P.run_gpu(lens, 256, 4, 2, 128, "bf16", seed=5, K=1)
    ref = P.run_oracle(lens, 4, 2, 128, "bf16", seed=5)
    P.check(b, ref, "bf16", "K=1")
    for sid in a:
        for n in ("o", "lse", "dq"):
            assert np.array_equal(a[sid][n], b[sid][n]), (sid, n)


@pytest.mark.parametrize("dtype,D,lens,C,Hq,Hkv", [
    ("bf16", 128, [1500, 40, 300, 77, 512, 129, 640, 9, 333, 200, 256, 31, 480, 64, 100, 700, 90, 411], 512, 8, 2),
    ("bf16", 128, [900, 40, 300], 256, 4, 2),
    ("fp32", 64, [700, 33, 1, 120, 64], 200, 2, 2),          # no MFMA path: the batch call falls back to single launches
])
def test_whole_plan_launch_matches_per_chunk_calls(dtype, D, lens, C, Hq, Hkv):
    """cf_attn_fwd_batch / cf_attn_bwd_batch (forward and dQ kernels of many chunks as one launch, more chunks
    than one launch holds in the first case) give what one call per chunk gives: O, LSE, dQ bit for bit, dK/dV
    to the parity tolerance (the heads of a group meet through atomic adds in both)."""
    a, _ = P.run_gpu(lens, C, Hq, Hkv, D, dtype, seed=7)
    b, eng = P.run_gpu(lens, C, Hq, Hkv, D, dtype, seed=7, fused_launch=True)
    assert eng.fused_launch and len(eng.chunks) >= 3
    ref = P.run_oracle(lens, Hq, Hkv, D, dtype, seed=7)
    print(len(eng.chunks), "chunks", P.check(b, ref, dtype, "whole-plan launch"))
    for sid in a:
        for n in ("o", "lse", "dq"):
            assert np.array_equal(a[sid][n], b[sid][n]), (sid, n)


def test_groups_dealt_over_streams_give_the_same_result():
    """The runner's multi-stream dispatch (groups on different streams, a workspace per stream, K = 1 schedule
    included) changes nothing: O, LSE, dQ bit for bit, dK/dV to the parity tolerance."""
    lens = [1500, 40, 300, 77, 512, 129, 640, 9, 333, 200, 256, 31, 480, 64]
    a, _ = P.run_gpu(lens, 512, 8, 2, 128, "bf16", seed=9)
    ref = P.run_oracle(lens, 8, 2, 128, "bf16", seed=9)
    for kw in (dict(n_streams=3), dict(n_streams=2, K=1)):
        b, eng = P.run_gpu(lens, 512, 8, 2, 128, "bf16", seed=9, **kw)
        assert len(eng.streams) == kw["n_streams"] and len({ch["lane"] for ch in eng.chunks}) == kw["n_streams"]
        P.check(b, ref, "bf16", f"streams {kw}")
        for sid in a:
            for n in ("o", "lse", "dq"):
                assert np.array_equal(a[sid][n], b[sid][n]), (kw, sid, n)


def test_strided_views_and_nonzero_initial_grads():
    """q/k/v as views into one packed buffer; dK/dV must be added to, dQ overwritten."""
    torch.manual_seed(0)
    dev = "cuda:0"
    T, Hq, Hkv, D = 300, 4, 2, 128
    qkv = torch.randn(T, Hq + 2 * Hkv, D, device=dev).to(torch.bfloat16)
    q, k, v = qkv[:, :Hq], qkv[:, Hq:Hq + Hkv], qkv[:, Hq + Hkv:]
    d_o = torch.randn(T, Hq, D, device=dev).to(torch.bfloat16)
    cu_host = np.array([0, 100, 101, 300], dtype=np.int32)
    cu = torch.from_numpy(cu_host).to(dev)
    o = torch.empty(T, Hq, D, device=dev, dtype=torch.bfloat16)
    lse = torch.empty(Hq, T, device=dev, dtype=torch.float32)
    scale = 1 / np.sqrt(D)
    fp = B.make_fwd_params(q, k, v, o, lse, cu, cu, scale)
    B.cf_attn_fwd(fp)
    dq = torch.full((T, Hq, D), 7.0, device=dev, dtype=torch.bfloat16)
    dkv0 = torch.randn(2, T, Hkv, D, device=dev)
    dkv = dkv0.clone()
    ws = torch.empty(B.cf_attn_bwd_workspace_bytes(fp), dtype=torch.uint8, device=dev)
    B.cf_attn_bwd(B.make_bwd_params(fp, d_o, dq, dkv[0], dkv[1], ws))
    torch.cuda.synchronize()
    f = lambda t: t.double().cpu().numpy()
    ro, rlse = OA.chunk_attn_fwd(f(q), f(k), f(v), cu_host, cu_host, np.float32(scale))
    rdk, rdv = np.zeros((T, Hkv, D)), np.zeros((T, Hkv, D))
    rdq = OA.chunk_attn_bwd(f(q), f(k), f(v), ro, rlse, f(d_o), cu_host, cu_host, np.float32(scale), rdk, rdv)
    got = {0: dict(o=f(o), lse=f(lse), dq=f(dq), dk=f(dkv[0] - dkv0[0]), dv=f(dkv[1] - dkv0[1]))}
    P.check(got, {0: dict(o=ro, lse=rlse, dq=rdq, dk=rdk, dv=rdv)}, "bf16", "strided")


def test_long_prefix_few_queries_fused_dkv_path():
    """A short slice (200 rows) behind a 65 400-token prefix: the dK/dV launch then has enough key tiles
    to fuse the query heads of a group into one workgroup (plain read-modify-write, no atomics)."""
    torch.manual_seed(1)
    dev = "cuda:0"
    T, P_, Hq, Hkv, D = 200, 65400, 16, 8, 128
    q = torch.randn(T, Hq, D, device=dev).to(torch.bfloat16)
    d_o = torch.randn(T, Hq, D, device=dev).to(torch.bfloat16)
    k = torch.randn(P_ + T, Hkv, D, device=dev).to(torch.bfloat16)
    v = torch.randn(P_ + T, Hkv, D, device=dev).to(torch.bfloat16)
    cu_q, cu_k = np.array([0, T], dtype=np.int32), np.array([0, P_ + T], dtype=np.int32)
    o = torch.empty_like(q)
    lse = torch.empty(Hq, T, device=dev, dtype=torch.float32)
    scale = 1 / np.sqrt(D)
    fp = B.make_fwd_params(q, k, v, o, lse, torch.from_numpy(cu_q).to(dev), torch.from_numpy(cu_k).to(dev), scale)
    B.cf_attn_fwd(fp)
    dq = torch.empty_like(q)
    dk = torch.zeros(P_ + T, Hkv, D, device=dev)
    dv = torch.zeros_like(dk)
    ws = torch.empty(B.cf_attn_bwd_workspace_bytes(fp), dtype=torch.uint8, device=dev)
    bp = B.make_bwd_params(fp, d_o, dq, dk, dv, ws)
    B.cf_attn_bwd(bp)
    torch.cuda.synchronize()
    f = lambda t: t.double().cpu().numpy()
    ro, rlse = OA.chunk_attn_fwd(f(q), f(k), f(v), cu_q, cu_k, np.float32(scale))
    rdk, rdv = np.zeros((P_ + T, Hkv, D)), np.zeros((P_ + T, Hkv, D))
    rdq = OA.chunk_attn_bwd(f(q), f(k), f(v), ro, rlse, f(d_o), cu_q, cu_k, np.float32(scale), rdk, rdv)
    got = {0: dict(o=f(o), lse=f(lse), dq=f(dq), dk=f(dk), dv=f(dv))}
    print(P.check(got, {0: dict(o=ro, lse=rlse, dq=rdq, dk=rdk, dv=rdv)}, "bf16", "long prefix"))
    dk2, dv2 = torch.zeros_like(dk), torch.zeros_like(dv)      # single writer per element: bitwise reproducible
    B.cf_attn_bwd(B.make_bwd_params(fp, d_o, dq, dk2, dv2, ws))
    torch.cuda.synchronize()
    assert torch.equal(dk, dk2) and torch.equal(dv, dv2)


def test_forward_and_dq_are_deterministic():
    """Forward and dQ have a single writer per element.  (dK/dV of short chunks sum the query heads of a
    group through fp32 atomics, so their last bits may differ between runs.)"""
    lens = [1500, 200, 77]
    a, _ = P.run_gpu(lens, 512, 8, 2, 128, "bf16", seed=6)
    b, _ = P.run_gpu(lens, 512, 8, 2, 128, "bf16", seed=6)
    for sid in a:
        for n in ("o", "lse", "dq"):
            assert np.array_equal(a[sid][n], b[sid][n]), (sid, n)


def test_device_entry_point_errors():
    dev = "cuda:0"
    q = torch.zeros(16, 2, 128, device=dev, dtype=torch.bfloat16)
    cu = torch.tensor([0, 16], device=dev, dtype=torch.int32)
    lse = torch.zeros(2, 16, device=dev)
    fp = B.make_fwd_params(q, q, q, q.clone(), lse, cu, cu, 0.1)
    ws = torch.empty(8, dtype=torch.uint8, device=dev)          # too small
    bp = B.make_bwd_params(fp, q, q.clone(), torch.zeros(16, 2, 128, device=dev), torch.zeros(16, 2, 128, device=dev), ws)
    with pytest.raises(B.CfError) as e:
        B.cf_attn_bwd(bp)
    assert e.value.code == B.CF_EINVAL and "workspace" in str(e.value)
    fp.q += 2                                                    # misaligned
    with pytest.raises(B.CfError):
        B.cf_attn_fwd(fp)


def test_fused_heads_dkv_accumulates_across_launches():
    """Section 4.2: earlier chunks rely on the key/value gradients of later chunks.  Three slices of one
    66 000-token sequence (8 key/value heads) run backward in DESCENDING order into one shared fp32 dK/dV state
    that starts non-zero.  Every launch has >= 4096 (key tile, kv head) pairs, so all three take the dK/dV
    kernel's fused-heads mode (plain read-modify-write) and add into the same prefix rows.  The WHOLE state is
    compared with the oracle's chunked backward applied in the same order, and a second run must reproduce the
    first bit for bit."""
    torch.manual_seed(3)
    dev = "cuda:0"
    L, T, Hq, Hkv, D = 66000, 200, 16, 8, 128
    starts = [65400, 65600, 65800]
    k = torch.randn(L, Hkv, D, device=dev).to(torch.bfloat16)
    v = torch.randn(L, Hkv, D, device=dev).to(torch.bfloat16)
    q = torch.randn(L - starts[0], Hq, D, device=dev).to(torch.bfloat16)        # rows of positions >= 65400
    d_o = torch.randn(L - starts[0], Hq, D, device=dev).to(torch.bfloat16)
    scale = 1 / np.sqrt(D)
    init = torch.randn(2, L, Hkv, D, device=dev) * 0.25
    f = lambda t: t.double().cpu().numpy()

    def run_gpu():
        dkv = init.clone()
        outs = []
        for P_ in reversed(starts):                                              # descending: last slice first
            a = P_ - starts[0]
            cu_q = torch.tensor([0, T], dtype=torch.int32, device=dev)
            cu_k = torch.tensor([0, P_ + T], dtype=torch.int32, device=dev)
            o = torch.empty(T, Hq, D, device=dev, dtype=torch.bfloat16)
            lse = torch.empty(Hq, T, device=dev, dtype=torch.float32)
            fp = B.make_fwd_params(q[a:a + T], k[:P_ + T], v[:P_ + T], o, lse, cu_q, cu_k, scale)
            assert (fp.n_kv_tokens // 128 + 1) * Hkv >= 4096                     # the fused-heads condition
            B.cf_attn_fwd(fp)
            dq = torch.empty(T, Hq, D, device=dev, dtype=torch.bfloat16)
            ws = torch.empty(B.cf_attn_bwd_workspace_bytes(fp), dtype=torch.uint8, device=dev)
            B.cf_attn_bwd(B.make_bwd_params(fp, d_o[a:a + T], dq, dkv[0][:P_ + T], dkv[1][:P_ + T], ws))
            outs.append((P_, o, lse, dq))
        torch.cuda.synchronize()
        return dkv, outs
    dkv, outs = run_gpu()
    # the oracle, same order, same non-zero start
    kk, vv = f(k), f(v)
    rdk, rdv = f(init[0]), f(init[1])
    max_abs, rel = P.TOL["bf16"]
    for P_, o, lse, dq in outs:
        a = P_ - starts[0]
        cu_q, cu_k = [0, T], [0, P_ + T]
        ro, rlse = OA.chunk_attn_fwd(f(q[a:a + T]), kk[:P_ + T], vv[:P_ + T], cu_q, cu_k, np.float32(scale))
        sdk, sdv = np.zeros((P_ + T, Hkv, D)), np.zeros((P_ + T, Hkv, D))
        rdq = OA.chunk_attn_bwd(f(q[a:a + T]), kk[:P_ + T], vv[:P_ + T], ro, rlse, f(d_o[a:a + T]), cu_q, cu_k,
                                np.float32(scale), sdk, sdv)
        rdk[:P_ + T] += sdk
        rdv[:P_ + T] += sdv
        got = {0: dict(o=f(o), lse=f(lse), dq=f(dq), dk=np.zeros(1), dv=np.zeros(1))}
        ref = {0: dict(o=ro, lse=rlse, dq=rdq, dk=np.zeros(1), dv=np.zeros(1))}
        print(f"slice at {P_}:", P.check(got, ref, "bf16", f"slice at {P_}"), flush=True)
    # the accumulated part alone (state minus its start), every row of the 66 000, against the oracle's
    for name, ours, theirs, start in (("dk", dkv[0], rdk, init[0]), ("dv", dkv[1], rdv, init[1])):
        got_c, ref_c = f(ours) - f(start), theirs - f(start)
        err = np.abs(got_c - ref_c).max()
        r2 = np.linalg.norm(got_c - ref_c) / np.linalg.norm(ref_c)
        # rows below the first slice received all three launches' contributions
        e3 = np.abs(got_c[:starts[0]] - ref_c[:starts[0]]).max()
        print(f"state {name}: max-abs {err:.2e} rel-L2 {r2:.2e} (prefix rows, three launches: {e3:.2e})", flush=True)
        assert err <= max_abs and r2 <= rel, (name, err, r2)
        assert np.abs(ref_c[:starts[0]]).max() > 0
    dkv2, _ = run_gpu()
    assert torch.equal(dkv, dkv2), "fused-heads dK/dV must be bitwise reproducible"


def test_single_writer_flag_makes_dkv_bitwise_reproducible():
    """CF_FLAG_DKV_SINGLE_WRITER: the dK/dV kernel's one-workgroup-per-key-tile mode on a small plan (long slices,
    packed short sequences, GQA 8/2): matches the oracle, and two runs agree bit for bit in ALL five tensors."""
    lens = [1500, 200, 77, 640, 129, 31]
    a, _ = P.run_gpu(lens, 512, 8, 2, 128, "bf16", seed=6, flags=B.CF_FLAG_DKV_SINGLE_WRITER)
    b, _ = P.run_gpu(lens, 512, 8, 2, 128, "bf16", seed=6, flags=B.CF_FLAG_DKV_SINGLE_WRITER)
    ref = P.run_oracle(lens, 8, 2, 128, "bf16", seed=6)
    print(P.check(a, ref, "bf16", "single-writer dK/dV"))
    for sid in a:
        for n in P.NAMES:
            assert np.array_equal(a[sid][n], b[sid][n]), (sid, n)
