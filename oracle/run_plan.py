"""ORACLE -- test infrastructure only: drive the chunked method over a whole plan on the CPU.

Forward passes run chunk by chunk with each dependency group in ascending order; backward passes
run with each group in descending order, adding key/value gradients into the per-sequence state
(paper section 4.2).  This is the all-activations-kept order (Algorithm 2 with N <= K).  The
result is returned per input sequence so that it can be compared with whole-sequence attention.
"""
import numpy as np

from . import attention as A


def run_plan(chunks, groups, seqs, scale):
    """seqs: {seq_id: dict(q [L,Hq,D], k [L,Hkv,D], v, d_o [L,Hq,D])} (any float dtype).

    Returns {seq_id: dict(o, lse [Hq,L], dq, dk, dv)} in fp64, computed chunk by chunk.
    """
    out = {}
    for sid, s in seqs.items():
        L, Hq, D = s["q"].shape
        Hkv = s["k"].shape[1]
        out[sid] = {"o": np.zeros((L, Hq, D)), "lse": np.zeros((Hq, L)), "dq": np.zeros((L, Hq, D)),
                    "dk": np.zeros((L, Hkv, D)), "dv": np.zeros((L, Hkv, D))}
    f64 = lambda a: np.asarray(a, dtype=np.float64)

    def gather(chunk):
        """Chunk-local query tensors, the key/value rows the chunk reads, and cu_seqlens."""
        qs, dos, ks, vs, cu_q, cu_k = [], [], [], [], [0], [0]
        for (sid, start, n) in chunk["segments"]:
            s = seqs[sid]
            qs.append(f64(s["q"][start:start + n]))
            dos.append(f64(s["d_o"][start:start + n]))
            ks.append(f64(s["k"][:start + n]))      # retained prefix state + own rows
            vs.append(f64(s["v"][:start + n]))
            cu_q.append(cu_q[-1] + n)
            cu_k.append(cu_k[-1] + start + n)
        return (np.concatenate(qs), np.concatenate(dos), np.concatenate(ks), np.concatenate(vs),
                np.array(cu_q), np.array(cu_k))

    for g in groups:
        for c in g["chunks"]:                      # ascending: later chunks read earlier state
            ch = chunks[c]
            q, _, k, v, cu_q, cu_k = gather(ch)
            o, lse = A.chunk_attn_fwd(q, k, v, cu_q, cu_k, scale)
            for n_seg, (sid, start, n) in enumerate(ch["segments"]):
                a, b = cu_q[n_seg], cu_q[n_seg + 1]
                out[sid]["o"][start:start + n] = o[a:b]
                out[sid]["lse"][:, start:start + n] = lse[:, a:b]
    for g in groups:
        for c in reversed(g["chunks"]):            # descending: prefix rows collect later chunks
            ch = chunks[c]
            q, d_o, k, v, cu_q, cu_k = gather(ch)
            o = np.concatenate([out[sid]["o"][st:st + n] for (sid, st, n) in ch["segments"]])
            lse = np.concatenate([out[sid]["lse"][:, st:st + n] for (sid, st, n) in ch["segments"]], axis=1)
            dk = np.concatenate([out[sid]["dk"][:st + n] for (sid, st, n) in ch["segments"]])
            dv = np.concatenate([out[sid]["dv"][:st + n] for (sid, st, n) in ch["segments"]])
            dq = A.chunk_attn_bwd(q, k, v, o, lse, d_o, cu_q, cu_k, scale, dk, dv)
            for n_seg, (sid, start, n) in enumerate(ch["segments"]):
                a, b = cu_q[n_seg], cu_q[n_seg + 1]
                ka, kb = cu_k[n_seg], cu_k[n_seg + 1]
                out[sid]["dq"][start:start + n] = dq[a:b]
                out[sid]["dk"][:start + n] = dk[ka:kb]
                out[sid]["dv"][:start + n] = dv[ka:kb]
    return out


def run_unsplit(seqs, scale):
    """Whole-sequence causal attention, one sequence at a time (the definition)."""
    out = {}
    for sid, s in seqs.items():
        o, lse = A.seq_attn_fwd(s["q"], s["k"], s["v"], scale)
        dq, dk, dv = A.seq_attn_bwd(s["q"], s["k"], s["v"], o, lse, s["d_o"], scale)
        out[sid] = {"o": o, "lse": lse, "dq": dq, "dk": dk, "dv": dv}
    return out
