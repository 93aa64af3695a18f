"""GPU parity at the FULL sizes of configs 2, 3, 4 and 5, in the launch configuration bench.py times (one
cf_attn_fwd / cf_attn_bwd call per chunk through the plan runner).  The fp64 oracle cannot redo these
sizes whole, so it recomputes sampled outputs one by one:
  - whole short sequences (all five tensors),
  - single query rows of the long (32768- / 262144-token) sequence (O, LSE, dQ; each needs only the keys before it),
  - dK/dV of the last keys of that sequence (they only depend on the last query rows).
"""
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


def host_values(cfg, seed, lens):
    HQ, HKV = inputs.CONFIGS[cfg]["Hq"], inputs.CONFIGS[cfg]["Hkv"]
    return lambda sid: inputs.seq_values(seed, sid, lens[sid], HQ, HKV, D, "bf16")


def device_values(cfg, seed, lens):
    """fp32 numpy views of values drawn on the device (the host generator needs minutes for config 5)."""
    HQ, HKV = inputs.CONFIGS[cfg]["Hq"], inputs.CONFIGS[cfg]["Hkv"]
    return lambda sid: inputs.seq_values_device(seed, sid, lens[sid], HQ, HKV, D, "bf16", "cuda:0")


def run_full(cfg, seed, on_device=False, pick_groups=None):
    """pick_groups(plan, lens) -> group ids to place and run (None: the whole plan)."""
    HQ, HKV = inputs.CONFIGS[cfg]["Hq"], inputs.CONFIGS[cfg]["Hkv"]

    def count(lens, C):
        p = B.cf_build_chunks(lens, C)
        n = p.n_chunks
        p.close()
        return n
    lens, C = inputs.seq_lens(cfg, seed, count)
    lens = [int(x) for x in lens]
    plan = B.cf_build_chunks(lens, C)
    values = (device_values if on_device else host_values)(cfg, seed, lens)
    only = pick_groups(plan, lens) if pick_groups else None
    eng = ChunkAttention(plan, HQ, HKV, D, "bf16", only_groups=only).load(lambda sid, L: values(sid))
    eng.zero_grads()
    eng.run_forward()
    eng.run_backward()
    torch.cuda.synchronize()
    return lens, C, plan, eng, values


def host(x):
    """fp32 numpy array of a generated tensor (numpy from the host generator, bf16 torch from the device one)."""
    return x.float().cpu().numpy() if torch.is_tensor(x) else x


def check_short_sequences(lens, plan, eng, values, picks):
    """All five tensors of whole short sequences against unsplit oracle attention."""
    HQ, HKV = eng.Hq, eng.Hkv
    where = {}
    for c, ch in enumerate(eng.chunks):
        if ch is not None and not ch["dependent"]:
            for i, (sid, start, n) in enumerate(ch["segs"]):
                where[sid] = (c, int(ch["cu_q_host"][i]), n)
    for sid in picks:
        c, a, n = where[sid]
        print(f"oracle: sequence {sid}, {n} tokens ...", flush=True)
        ch = eng.chunks[c]
        v = {k: host(x) for k, x in values(sid).items()}
        o, lse = OA.seq_attn_fwd(v["q"], v["k"], v["v"], SCALE)
        dq, dk, dv = OA.seq_attn_bwd(v["q"], v["k"], v["v"], o, lse, v["d_o"], SCALE)
        got = {0: dict(o=f64(ch["o"][a:a + n]), lse=f64(ch["lse"][:, a:a + n]), dq=f64(ch["d_q"][a:a + n]),
                       dk=f64(ch["dk"][a:a + n]), dv=f64(ch["dv"][a:a + n]))}
        errs = P.check(got, {0: dict(o=o, lse=lse, dq=dq, dk=dk, dv=dv)}, "bf16", f"sequence {sid} (len {n})")
        print(f"seq {sid} len {n}:", {k: f"{e[0]:.2e}/{e[1]:.2e}" for k, e in errs.items()}, flush=True)


def test_config2_full_size_sampled_sequences():
    lens, C, plan, eng, values = run_full("packed_8k", 0)
    assert plan.n_chunks == 16 and C == 8192
    order = np.argsort(lens)
    picks = [int(order[0]), int(order[len(order) // 4]), int(order[len(order) // 2]), int(order[-8])]
    check_short_sequences(lens, plan, eng, values, picks)


def check_long_sequence(lens, C, eng, values, rows, W, sid=0):
    """Sampled query rows (O, LSE, dQ) and the dK/dV of the last W keys of the split sequence sid."""
    HQ, HKV = eng.Hq, eng.Hkv
    L = lens[sid]
    dev = values(sid)
    # the oracle needs every key and value, but only the sampled rows of q and d_o
    v = {"k": host(dev["k"]), "v": host(dev["v"])}
    take = sorted(set(rows) | set(range(L - W, L)))
    at = {r: n for n, r in enumerate(take)}
    idx = take if not torch.is_tensor(dev["q"]) else torch.tensor(take, device=dev["q"].device)
    q_s, do_s = host(dev["q"][idx]), host(dev["d_o"][idx])
    del dev
    g = [x for x in range(eng.plan.n_groups) if int(eng.plan.group_seq_id[x]) == sid][0]
    group_chunks = eng.plan.group(g)
    got = {"o": [], "lse": [], "dq": []}
    ref = {"o": [], "lse": [], "dq": []}
    for r in rows:
        c, i = r // C, r % C
        ch = eng.chunks[group_chunks[c]]
        assert ch["dependent"] and ch["P"] == c * C
        n = at[r]
        o, lse = OA.chunk_attn_fwd(q_s[n:n + 1], v["k"][:r + 1], v["v"][:r + 1], [0, 1], [0, r + 1], SCALE)
        dk = np.zeros((r + 1, HKV, D)); dv = np.zeros((r + 1, HKV, D))
        dq = OA.chunk_attn_bwd(q_s[n:n + 1], v["k"][:r + 1], v["v"][:r + 1], o, lse, do_s[n:n + 1],
                               [0, 1], [0, r + 1], SCALE, dk, dv)
        ref["o"].append(o); ref["lse"].append(lse); ref["dq"].append(dq)
        got["o"].append(f64(ch["o"][i:i + 1])); got["lse"].append(f64(ch["lse"][:, i:i + 1])); got["dq"].append(f64(ch["d_q"][i:i + 1]))
    max_abs, rel = P.TOL["bf16"]
    for name in got:
        a, b = np.concatenate(got[name], axis=-2 if name != "lse" else -1), np.concatenate(ref[name], axis=-2 if name != "lse" else -1)
        err, r2 = np.abs(a - b).max(), np.linalg.norm(a - b) / np.linalg.norm(b)
        print(f"rows {name}: max-abs {err:.2e} rel-L2 {r2:.2e}", flush=True)
        assert err <= max_abs and r2 <= rel, (name, err, r2)
    # ---- dK/dV of the last W keys: complete once the last W query rows (all in the last chunk) are done
    qs, dos = q_s[at[L - W]:], do_s[at[L - W]:]
    o, lse = OA.chunk_attn_fwd(qs, v["k"], v["v"], [0, W], [0, L], SCALE)
    dk = np.zeros((L, HKV, D)); dv = np.zeros((L, HKV, D))
    OA.chunk_attn_bwd(qs, v["k"], v["v"], o, lse, dos, [0, W], [0, L], SCALE, dk, dv)
    st = eng.state[g]
    for name, ours, theirs in (("dk", st["dk"], dk), ("dv", st["dv"], dv)):
        a, b = f64(ours[L - W:]), theirs[L - W:]
        err, r2 = np.abs(a - b).max(), np.linalg.norm(a - b) / np.linalg.norm(b)
        print(f"tail keys {name}: max-abs {err:.2e} rel-L2 {r2:.2e}", flush=True)
        assert err <= max_abs and r2 <= rel, (name, err, r2)


def test_config3_full_size_sampled_rows_and_tail_keys():
    lens, C, plan, eng, values = run_full("long32k_mixed", 0)
    assert plan.n_chunks == 12 and lens[0] == 32768
    L = lens[0]
    # single query rows: chunk boundaries, tile edges, the very last row
    check_long_sequence(lens, C, eng, values, [0, 1, 127, 8191, 8192, 8193, 16383 + 64, 24576, 24576 + 4095, L - 1], 160)
    # ---- and a few of the packed short sequences of the same batch
    order = np.argsort(lens[1:]) + 1
    check_short_sequences(lens, plan, eng, values, [int(order[1]), int(order[len(order) // 2])])


def test_config5_full_size_sampled_rows_and_tail_keys():
    """One 262144-token sequence in 8 chunks of 32768 (prefix state up to 229376 rows), 64 / 8 heads."""
    lens, C, plan, eng, values = run_full("long256k_32k", 0, on_device=True)
    assert plan.n_chunks == 12 and lens[0] == 262144 and C == 32768
    L = lens[0]
    check_long_sequence(lens, C, eng, values, [0, 32767, 32768, 131072 + 63, 229376, 229376 + 12345, L - 1], 32)
    order = np.argsort(lens[1:]) + 1
    check_short_sequences(lens, plan, eng, values, [int(order[1]), int(order[len(order) // 2])])


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
    for which, W in (("longest", 24), ("shortest", 64)):
        sid = int(plan.group_seq_id[picked[which]])
        L = lens[sid]
        n_slices = -(-L // C)
        assert len(plan.group(picked[which])) == n_slices
        rows = sorted({0, C - 1, C, (n_slices - 1) * C, max(0, (n_slices - 1) * C - 1), L - 1, L // 2})
        print(f"{which} split sequence {sid}: {L} tokens, {n_slices} slices", flush=True)
        check_long_sequence(lens, C, eng, values, rows, min(W, L - (n_slices - 1) * C), sid=sid)
    # whole short sequences of the two packed chunks (the oracle redoes each alone: keep them under 2000 tokens)
    shorts = []
    for g in picked["packed"]:
        segs = [x for x in eng.chunks[plan.group(g)[0]]["segs"] if x[2] <= 2000]
        by_len = sorted(segs, key=lambda x: x[2])
        shorts += [by_len[0][0], by_len[len(by_len) // 2][0], by_len[-1][0]]
    check_short_sequences(lens, plan, eng, values, shorts)
