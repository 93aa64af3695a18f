"""GPU parity at the FULL sizes of configs 2, 3, 4 and 5, in the launch configuration bench.py times (one
cf_attn_fwd / cf_attn_bwd call per chunk through the plan runner).

What the fp64 oracle recomputes, per config (every check uses the benchmark spec's tolerance of tests/parity.py):
  config 2  all 167 sequences, all five tensors (O, LSE, dQ, dK, dV), element by element.
  config 3  every packed short sequence, all five tensors; for the 32768-token sequence the whole of O, LSE, dQ of
            query heads 0-6 and the whole of dK, dV of key/value head 0 over all 32768 keys (inputs sliced to that
            one GQA group: key/value head 0's gradients only collect from query heads 0-6) -- rows [0, 24576) of
            that state were added into by up to four backward launches -- plus 16 rows per chunk over all four GQA groups.
  config 5  64 query rows of EVERY dependent chunk, as 4 runs of 16 consecutive rows (the chunk's first 16, its last
            16 and two seeded random runs): O, LSE, dQ on one GQA group per run (the key/value head rotates from run
            to run, so the 32 runs cover all 64 query heads 4 times; runs, because the oracle spreads the rows of ONE
            call over the host cores, and one group, because a row over all heads costs it 8 times as much); dK, dV of the last 1024 keys for key/value head 0 (they depend only on the
            last 1024 query rows of query heads 0-7); whole random short sequences of the packed chunks, all five
            tensors; and a GPU-vs-GPU run of the long sequence at ChunkSize 32768 and 16384 over all rows and all
            five tensors (chunk-size independence of the method).
  config 4  the 20000-sequence batch is planned whole; the longest and the shortest split sequence and two packed
            chunks are placed and run; checks as for config 5 (64 rows per dependent chunk in 4 runs, 1024-key tail for
            key/value head 0, whole short sequences, ChunkSize 16384 vs 8192 on the longest split sequence).
"""
import time

import numpy as np
import pytest
import torch

from oracle import attention as OA
from paper_2503_02356_amd import binding as B
from paper_2503_02356_amd import inputs
from paper_2503_02356_amd.runner import ChunkAttention
from tests import parity as P

pytestmark = pytest.mark.gpu
D = 128
SCALE = np.float32(1.0 / np.sqrt(D))
f64 = lambda t: t.detach().to(torch.float64).cpu().numpy()
MAX_ABS, REL = P.TOL["bf16"]


def host_values(cfg, seed, lens):
    HQ, HKV = inputs.CONFIGS[cfg]["Hq"], inputs.CONFIGS[cfg]["Hkv"]
    return lambda sid: inputs.seq_values(seed, sid, lens[sid], HQ, HKV, D, "bf16")


def device_values(cfg, seed, lens):
    """Values drawn on the device (the host generator needs minutes for config 5)."""
    HQ, HKV = inputs.CONFIGS[cfg]["Hq"], inputs.CONFIGS[cfg]["Hkv"]
    return lambda sid: inputs.seq_values_device(seed, sid, lens[sid], HQ, HKV, D, "bf16", "cuda:0")


def count_chunks(lens, C):
    p = B.cf_build_chunks(lens, C)
    n = p.n_chunks
    p.close()
    return n


def run_full(cfg, seed, on_device=False, pick_groups=None):
    """pick_groups(plan, lens) -> group ids to place and run (None: the whole plan)."""
    HQ, HKV = inputs.CONFIGS[cfg]["Hq"], inputs.CONFIGS[cfg]["Hkv"]
    lens, C = inputs.seq_lens(cfg, seed, count_chunks)
    lens = [int(x) for x in lens]
    plan = B.cf_build_chunks(lens, C)
    values = (device_values if on_device else host_values)(cfg, seed, lens)
    only = pick_groups(plan, lens) if pick_groups else None
    eng = ChunkAttention(plan, HQ, HKV, D, "bf16", only_groups=only).load(lambda sid, L: values(sid))
    eng.zero_grads()
    eng.run_forward()
    eng.run_backward()
    torch.cuda.synchronize()
    P.progress(f"{cfg}: {plan.n_chunks} chunks planned, forward + backward done on the GPU")
    return lens, C, plan, eng, values


def host(x):
    """fp64 numpy array of a generated tensor (numpy from the host generator, bf16 torch from the device one)."""
    return x.double().cpu().numpy() if torch.is_tensor(x) else np.asarray(x, dtype=np.float64)


class Errors:
    """Max-abs and relative-L2 error per tensor name, accumulated over many pieces."""

    def __init__(self):
        self.acc = {}

    def add(self, name, got, ref):
        d = got - ref
        a = self.acc.setdefault(name, [0.0, 0.0, 0.0, 0])
        a[0] = max(a[0], float(np.abs(d).max()))
        a[1] += float((d * d).sum())
        a[2] += float((ref * ref).sum())
        a[3] += d.size

    def check(self, what):
        for name, (mx, num, den, n) in self.acc.items():
            rel = np.sqrt(num / den) if den > 0 else 0.0
            P.progress(f"{what} {name}: {n} elements, max-abs {mx:.2e} rel-L2 {rel:.2e}")
            assert np.isfinite(mx) and mx <= MAX_ABS and rel <= REL, (what, name, mx, rel)


def check_short_sequences(eng, values, picks, what):
    """All five tensors of whole short sequences against unsplit oracle attention."""
    where = {}
    for c, ch in enumerate(eng.chunks):
        if ch is not None and not ch["dependent"]:
            for i, (sid, start, n) in enumerate(ch["segs"]):
                where[sid] = (c, int(ch["cu_q_host"][i]), n)
    errs = Errors()
    t0 = time.time()
    for n_done, sid in enumerate(picks):
        c, a, n = where[sid]
        ch = eng.chunks[c]
        v = {k: host(x) for k, x in values(sid).items()}
        o, lse = OA.seq_attn_fwd(v["q"], v["k"], v["v"], SCALE)
        dq, dk, dv = OA.seq_attn_bwd(v["q"], v["k"], v["v"], o, lse, v["d_o"], SCALE)
        got = dict(o=f64(ch["o"][a:a + n]), lse=f64(ch["lse"][:, a:a + n]), dq=f64(ch["d_q"][a:a + n]),
                   dk=f64(ch["dk"][a:a + n]), dv=f64(ch["dv"][a:a + n]))
        one = Errors()
        for name, ref in (("o", o), ("lse", lse), ("dq", dq), ("dk", dk), ("dv", dv)):
            errs.add(name, got[name], ref)
            one.add(name, got[name], ref)
        for name, (mx, num, den, _) in one.acc.items():     # the bound holds for every sequence on its own, too
            rel = np.sqrt(num / den) if den > 0 else 0.0
            assert mx <= MAX_ABS and rel <= REL, (what, "sequence", sid, "len", n, name, mx, rel)
        if (n_done + 1) % 20 == 0 or n_done + 1 == len(picks):
            P.progress(f"{what}: {n_done + 1}/{len(picks)} sequences checked, {time.time() - t0:.0f} s")
    errs.check(what)


def test_config2_full_size_all_sequences():
    lens, C, plan, eng, values = run_full("packed_8k", 0)
    assert plan.n_chunks == 16 and C == 8192
    check_short_sequences(eng, values, list(range(len(lens))), f"config 2, all {len(lens)} sequences")


def split_group(eng, sid):
    return [g for g in range(eng.plan.n_groups) if int(eng.plan.group_seq_id[g]) == sid][0]


def sample_runs(rng, eng, g, n_runs, run_len):
    """n_runs runs of run_len consecutive query rows in EVERY chunk of group g, as (first global row, length): one at
    the chunk's first row, one ending at its last row, the others at seeded random places.  (Runs, not single rows:
    the oracle spreads the rows of one call over the host cores.)"""
    runs = []
    for c in eng.plan.group(g):
        ch = eng.chunks[c]
        T, P_ = ch["T"], ch["P"]
        n = min(run_len, T)
        starts = {0, T - n} | {int(x) for x in rng.integers(0, T - n + 1, size=max(0, n_runs - 2))}
        runs += [(P_ + a, n) for a in sorted(starts)]
    return runs


def per_kv_head(x64):
    """[L, Hkv, D] -> list of contiguous [L, 1, D] arrays (the oracle then streams one head's rows)."""
    return [np.ascontiguousarray(x64[:, h:h + 1]) for h in range(x64.shape[1])]


def check_rows(eng, g, C, k_heads, v_heads, q_of, do_of, runs, what):
    """O, LSE, dQ of runs of query rows: a run [a, a+n) needs only the keys [0, a+n).  Run number m is checked on
    the query heads of key/value head m % Hkv (the inputs sliced to that one GQA group, whose outputs depend on
    nothing else), so the runs cover all heads between them."""
    chunks = eng.plan.group(g)
    Hkv, G = eng.Hkv, eng.Hq // eng.Hkv
    errs = Errors()
    scratch_k, scratch_v = np.zeros_like(k_heads[0]), np.zeros_like(k_heads[0])   # the oracle's dK/dV output, not looked at
    t0, n_rows = time.time(), 0
    for m, (a, n) in enumerate(runs):
        ch = eng.chunks[chunks[a // C]]
        i = a - ch["P"]
        assert 0 <= i and i + n <= ch["T"]
        kh = m % Hkv
        hs = slice(kh * G, (kh + 1) * G)
        q_r, do_r = np.ascontiguousarray(q_of(a, n)[:, hs]), np.ascontiguousarray(do_of(a, n)[:, hs])
        k_r, v_r = k_heads[kh][:a + n], v_heads[kh][:a + n]
        o, lse = OA.chunk_attn_fwd(q_r, k_r, v_r, [0, n], [0, a + n], SCALE)
        dq = OA.chunk_attn_bwd(q_r, k_r, v_r, o, lse, do_r, [0, n], [0, a + n], SCALE, scratch_k[:a + n], scratch_v[:a + n])
        errs.add("o", f64(ch["o"][i:i + n, hs]), o)
        errs.add("lse", f64(ch["lse"][hs, i:i + n]), lse)
        errs.add("dq", f64(ch["d_q"][i:i + n, hs]), dq)
        n_rows += n
        if (m + 1) % 8 == 0 or m + 1 == len(runs):
            P.progress(f"{what}: {n_rows} rows in {m + 1}/{len(runs)} runs checked, {time.time() - t0:.0f} s")
    errs.check(what)


def check_tail_keys(eng, g, k0, v0, q_tail, do_tail, W, G, what):
    """dK, dV of the last W keys of key/value head 0 (k0, v0: its [L, 1, D] rows): they depend only on the last W
    query rows of its G query heads."""
    L = k0.shape[0]
    qs, dos = np.ascontiguousarray(q_tail[:, :G]), np.ascontiguousarray(do_tail[:, :G])
    P.progress(f"{what}: oracle ...")
    o, lse = OA.chunk_attn_fwd(qs, k0, v0, [0, W], [0, L], SCALE)
    dk, dv = np.zeros((L, 1, D)), np.zeros((L, 1, D))
    OA.chunk_attn_bwd(qs, k0, v0, o, lse, dos, [0, W], [0, L], SCALE, dk, dv)
    st = eng.state[g]
    errs = Errors()
    errs.add("dk", f64(st["dk"][L - W:, :1]), dk[L - W:])
    errs.add("dv", f64(st["dv"][L - W:, :1]), dv[L - W:])
    errs.check(what)


def rerun_with_chunk_size(values, sid, L, HQ, HKV, C2):
    """The split sequence alone, chunked at C2, forward + backward on the GPU: per-sequence results on the device."""
    plan = B.cf_build_chunks([L], C2)
    eng = ChunkAttention(plan, HQ, HKV, D, "bf16").load(lambda s, n: values(sid))
    eng.zero_grads()
    eng.run_forward()
    eng.run_backward()
    torch.cuda.synchronize()
    return plan, eng


def check_chunk_size_independence(eng, g, values, sid, L, C, what):
    """GPU vs GPU: the same sequence chunked at C and at C/2 (all rows, all heads, all five tensors).  Both are
    within the tolerance of the exact result, so they differ by at most twice that."""
    HQ, HKV = eng.Hq, eng.Hkv
    P.progress(f"{what}: second GPU run ...")
    plan2, eng2 = rerun_with_chunk_size(values, sid, L, HQ, HKV, C // 2)
    assert plan2.n_chunks == -(-L // (C // 2))
    st, st2 = eng.state[g], eng2.state[0]
    diff = lambda a, b: (float((a.double() - b.double()).abs().max()),
                         float(torch.linalg.vector_norm(a.double() - b.double()) / torch.linalg.vector_norm(b.double())))
    out = {"dk": diff(st["dk"], st2["dk"]), "dv": diff(st["dv"], st2["dv"])}
    cat = lambda e, chunks, key, dim: torch.cat([e.chunks[c][key] for c in chunks], dim=dim)
    a_chunks, b_chunks = eng.plan.group(g), eng2.plan.group(0)
    for name, key, dim in (("o", "o", 0), ("dq", "d_q", 0), ("lse", "lse", 1)):
        out[name] = diff(cat(eng, a_chunks, key, dim), cat(eng2, b_chunks, key, dim))
    P.progress(what, {k: f"{v[0]:.2e}/{v[1]:.2e}" for k, v in out.items()})
    for name, (mx, rel) in out.items():
        assert mx <= 2 * MAX_ABS and rel <= 2 * REL, (what, name, mx, rel)
    del eng2


def check_split_sequence(eng, values, sid, L, C, rng, what, n_runs=4, run_len=16, W=1024, self_consistency=True):
    HQ, HKV = eng.Hq, eng.Hkv
    g = split_group(eng, sid)
    dev = values(sid)
    k_heads, v_heads = per_kv_head(host(dev["k"])), per_kv_head(host(dev["v"]))
    runs = sample_runs(rng, eng, g, n_runs, run_len)
    q_of = lambda a, n: host(dev["q"][a:a + n])
    do_of = lambda a, n: host(dev["d_o"][a:a + n])
    check_rows(eng, g, C, k_heads, v_heads, q_of, do_of, runs, f"{what}: {n_runs * run_len} rows per dependent chunk")
    W = min(W, L)
    check_tail_keys(eng, g, k_heads[0], v_heads[0], host(dev["q"][L - W:]), host(dev["d_o"][L - W:]), W, HQ // HKV,
                    f"{what}: last {W} keys, kv head 0")
    del k_heads, v_heads
    if self_consistency:
        check_chunk_size_independence(eng, g, values, sid, L, C, f"{what}: ChunkSize {C} vs {C // 2}")


def test_config3_full_size_long_sequence_group_and_all_packed_sequences():
    lens, C, plan, eng, values = run_full("long32k_mixed", 0)
    assert plan.n_chunks == 12 and lens[0] == 32768
    L, HQ, HKV = lens[0], eng.Hq, eng.Hkv
    G = HQ // HKV
    g = split_group(eng, 0)
    v = {k: host(x) for k, x in values(0).items()}
    # ---- one whole GQA group of the long sequence: query heads 0..G-1, key/value head 0, every row and key
    t0 = time.time()
    sl = {"q": v["q"][:, :G], "d_o": v["d_o"][:, :G], "k": v["k"][:, :1], "v": v["v"][:, :1]}
    sl = {k: np.ascontiguousarray(x) for k, x in sl.items()}
    # (in two calls, heads 0-3 and 4-6: dK and dV of the key/value head are the sums over its query heads, and a
    # progress line appears every minute or so)
    o, lse, dq = np.empty_like(sl["q"]), np.empty((G, L)), np.empty_like(sl["q"])
    dk, dv = np.zeros_like(sl["k"]), np.zeros_like(sl["k"])
    for h0, h1 in ((0, 4), (4, G)):
        qs, dos = np.ascontiguousarray(sl["q"][:, h0:h1]), np.ascontiguousarray(sl["d_o"][:, h0:h1])
        o_p, lse_p = OA.seq_attn_fwd(qs, sl["k"], sl["v"], SCALE)
        P.progress(f"oracle forward, heads {h0}-{h1 - 1}: {time.time() - t0:.0f} s; backward ...")
        dq_p, dk_p, dv_p = OA.seq_attn_bwd(qs, sl["k"], sl["v"], o_p, lse_p, dos, SCALE)
        o[:, h0:h1], lse[h0:h1], dq[:, h0:h1] = o_p, lse_p, dq_p
        dk += dk_p
        dv += dv_p
        P.progress(f"oracle: 32768-token sequence, heads {h0}-{h1 - 1}: {time.time() - t0:.0f} s")
    chunks = plan.group(g)
    assert [eng.chunks[c]["P"] for c in chunks] == [0, 8192, 16384, 24576]
    errs = Errors()
    for c in chunks:
        ch = eng.chunks[c]
        a, b = ch["P"], ch["P"] + ch["T"]
        errs.add("o", f64(ch["o"][:, :G]), o[a:b])
        errs.add("dq", f64(ch["d_q"][:, :G]), dq[a:b])
        errs.add("lse", f64(ch["lse"][:G]), lse[:, a:b])
    st = eng.state[g]
    errs.add("dk", f64(st["dk"][:, :1]), dk)
    errs.add("dv", f64(st["dv"][:, :1]), dv)
    # the prefix rows alone (four launches added into rows [0, 8192), three into the next 8192, ...)
    errs.add("dk rows [0, 24576)", f64(st["dk"][:24576, :1]), dk[:24576])
    errs.add("dv rows [0, 24576)", f64(st["dv"][:24576, :1]), dv[:24576])
    errs.check("config 3, long sequence, GQA group 0")
    # ---- 16 random rows over ALL heads
    rng = np.random.default_rng(33)
    runs = sample_runs(rng, eng, g, 4, 4)
    check_rows(eng, g, C, per_kv_head(v["k"]), per_kv_head(v["v"]), lambda a, n: v["q"][a:a + n], lambda a, n: v["d_o"][a:a + n],
               runs, "config 3, long sequence, 16 rows per chunk over all four GQA groups")
    # ---- every packed short sequence of the batch
    check_short_sequences(eng, values, list(range(1, len(lens))), f"config 3, all {len(lens) - 1} packed sequences")


def test_config5_full_size_rows_tail_keys_short_sequences_and_chunk_size_independence():
    """One 262144-token sequence in 8 chunks of 32768 (prefix state up to 229376 rows), 64 / 8 heads."""
    lens, C, plan, eng, values = run_full("long256k_32k", 0, on_device=True)
    assert plan.n_chunks == 12 and lens[0] == 262144 and C == 32768
    rng = np.random.default_rng(55)
    check_split_sequence(eng, values, 0, lens[0], C, rng, "config 5")
    picks = [int(x) for x in rng.choice(np.arange(1, len(lens)), size=6, replace=False)]
    check_short_sequences(eng, values, picks, "config 5, random short sequences")


def test_config4_full_size_sampled_groups():
    """The 20000-sequence long-tail batch (32 / 8 heads, chunk 16384) is planned whole; its tensors do not fit one
    GPU at once, so the groups are run a few at a time as a training loop would: here the longest split sequence,
    the shortest split sequence and two packed chunks (a middle one and the last), each checked against the oracle."""
    cfg = "longtail_16k"
    picked = {}

    def pick(plan, lens):
        split = sorted((lens[int(plan.group_seq_id[g])], g) for g in range(plan.n_groups) if int(plan.group_seq_id[g]) >= 0)
        packed = [g for g in range(plan.n_groups) if int(plan.group_seq_id[g]) < 0]
        mid = packed[len(packed) // 2]      # (the first packed chunks hold one ChunkSize-long sequence each)
        picked.update(longest=split[-1][1], shortest=split[0][1], packed=[mid, packed[-1]])
        return [split[-1][1], split[0][1], mid, packed[-1]]
    lens, C, plan, eng, values = run_full(cfg, 0, on_device=True, pick_groups=pick)
    assert len(lens) == 20000 and C == 16384 and plan.n_chunks > 900
    rng = np.random.default_rng(44)
    for which in ("longest", "shortest"):
        sid = int(plan.group_seq_id[picked[which]])
        L = lens[sid]
        n_slices = -(-L // C)
        assert len(plan.group(picked[which])) == n_slices
        P.progress(f"{which} split sequence {sid}: {L} tokens, {n_slices} slices")
        check_split_sequence(eng, values, sid, L, C, rng, f"config 4, {which} split sequence ({L} tokens)",
                             self_consistency=which == "longest")
    # whole short sequences of the two packed chunks (the oracle redoes each alone: keep them under 2000 tokens)
    shorts = []
    for g in picked["packed"]:
        segs = [x for x in eng.chunks[plan.group(g)[0]]["segs"] if x[2] <= 2000]
        take = rng.choice(len(segs), size=min(4, len(segs)), replace=False)
        shorts += [segs[int(i)][0] for i in take]
    check_short_sequences(eng, values, shorts, "config 4, random short sequences")
