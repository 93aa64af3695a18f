"""Algorithm 2 executed with a bounded activation pool (paper section 4.2, table 5's memory trend).

The plan runner (runner.py) keeps every chunk's tensors on the GPU for the whole step, which is what a timing
run wants.  This executor instead holds on the GPU only what Algorithm 2 says must be held:

  * K activation slots (query rows, attention output, log-sum-exp of one chunk each): a FWD_KEEP op takes a slot
    and its chunk's BWD op gives it back; more than K never exist;
  * one scratch slot that a FWD_DISCARD op writes into and that is poisoned (NaN) as soon as the op is done, so
    that nothing can use a discarded chunk's activations afterwards: its backward is only possible after the
    second forward that Algorithm 2 schedules;
  * the key/value state of the split sequence being processed and its fp32 gradient state (both live from the
    group's first op to its last and start out poisoned resp. zero: a chunk's key/value rows enter the state when
    its FIRST forward runs, in ascending order, as section 4.2 requires);
  * one chunk's worth of transient buffers (output gradient, query gradient; keys, values and their gradients of
    a standalone chunk) and the backward workspace.

Everything else -- the chunk inputs a model's other layers would produce on the fly, and the results they would
consume -- lives in pinned host memory and crosses to the GPU only for the op that needs it.  Memory placement
and launch order only: every arithmetic step runs inside cf_attn_fwd / cf_attn_bwd.

Chunks that hold a merged tail (cf_build_chunks_ex with CF_PLAN_MERGE_TAILS) are not supported here.
"""
import numpy as np
import torch

from . import binding as B


class _Slot:
    def __init__(self, C, Hq, D, dtype, dev):
        self.q = torch.empty((C, Hq, D), dtype=dtype, device=dev)
        self.o = torch.empty((C, Hq, D), dtype=dtype, device=dev)
        self.lse = torch.empty(Hq * C, dtype=torch.float32, device=dev)
        self.chunk = None

    def poison(self):
        self.q.fill_(float("nan"))
        self.o.fill_(float("nan"))
        self.lse.fill_(float("nan"))
        self.chunk = None

    def bytes(self):
        return sum(t.numel() * t.element_size() for t in (self.q, self.o, self.lse))


class SlotExecutor:
    def __init__(self, plan, n_q_heads, n_kv_heads, head_dim, dtype, K, scale=None, device="cuda:0", flags=0):
        self.plan, self.Hq, self.Hkv, self.D, self.K = plan, n_q_heads, n_kv_heads, head_dim, int(K)
        self.tdtype = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.scale = float(scale) if scale is not None else 1.0 / float(np.sqrt(head_dim))
        self.dev, self.flags = torch.device(device), flags
        for c in range(plan.n_chunks):
            if int(plan.group_seq_id[int(plan.chunk_group[c])]) >= 0 and len(plan.chunk_segments(c)) > 1:
                raise NotImplementedError("chunks with a merged tail are not supported by SlotExecutor")
        self.host = {}          # chunk id -> pinned host tensors: inputs q, k, v, d_o and results o, lse, d_q
        self.host_state = {}    # group id -> pinned dk, dv results of a split sequence
        self.peak_slots = 0
        self.n_forward = self.n_backward = 0

    # ------------------------------------------------------------------ host side ("the other layers")
    def load(self, values):
        """values(seq_id, L) -> dict(q, k, v, d_o) of fp32 numpy arrays [L, H, D] (representable in the compute
        dtype).  Everything is stored in pinned host memory, per chunk."""
        p, dt = self.plan, self.tdtype
        pin = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dt).pin_memory()
        seq_len = {}
        for s in range(p.n_segments):
            sid = int(p.seg_seq_id[s])
            seq_len[sid] = max(seq_len.get(sid, 0), int(p.seg_seq_start[s]) + int(p.seg_len[s]))
        cache = {}

        def get(sid):
            if sid not in cache:
                cache.clear()
                cache[sid] = values(sid, seq_len[sid])
            return cache[sid]
        for c in range(p.n_chunks):
            parts = {n: [] for n in ("q", "k", "v", "d_o")}
            for sid, start, n in p.chunk_segments(c):
                v = get(sid)
                for name in parts:
                    parts[name].append(v[name][start:start + n])
            h = {name: pin(np.concatenate(parts[name], axis=0)) for name in parts}
            T = int(p.chunk_tokens[c])
            h["o"] = torch.empty((T, self.Hq, self.D), dtype=dt).pin_memory()
            h["d_q"] = torch.empty((T, self.Hq, self.D), dtype=dt).pin_memory()
            h["lse"] = torch.empty((self.Hq, T), dtype=torch.float32).pin_memory()
            g = int(p.chunk_group[c])
            if int(p.group_seq_id[g]) < 0:
                h["dk"] = torch.empty((T, self.Hkv, self.D), dtype=torch.float32).pin_memory()
                h["dv"] = torch.empty((T, self.Hkv, self.D), dtype=torch.float32).pin_memory()
            self.host[c] = h
        self.seq_len = seq_len
        return self

    # ------------------------------------------------------------------ device side
    def _allocate(self):
        p, dev, dt = self.plan, self.dev, self.tdtype
        C = int(max(p.chunk_tokens)) if p.n_chunks else 1
        self.C = C
        self.slots = [_Slot(C, self.Hq, self.D, dt, dev) for _ in range(self.K)]
        self.scratch = _Slot(C, self.Hq, self.D, dt, dev)
        for s in self.slots + [self.scratch]:
            s.poison()
        self.d_o = torch.empty((C, self.Hq, self.D), dtype=dt, device=dev)
        self.d_q = torch.empty((C, self.Hq, self.D), dtype=dt, device=dev)
        self.kv = torch.empty((2, C, self.Hkv, self.D), dtype=dt, device=dev)          # a standalone chunk's own K, V
        self.dkv = torch.empty((2, C, self.Hkv, self.D), dtype=torch.float32, device=dev)
        self.cu = {}
        for c in range(p.n_chunks):
            cu = p.chunk_cu_seqlens(c)
            P, T = int(p.chunk_prefix_len[c]), int(p.chunk_tokens[c])
            dependent = int(p.group_seq_id[int(p.chunk_group[c])]) >= 0
            cu_k = np.array([0, P + T], dtype=np.int32) if dependent else cu
            self.cu[c] = (torch.from_numpy(cu.copy()).to(dev), torch.from_numpy(cu_k.copy()).to(dev))
        self.workspace = None
        self._ws_bytes = 0
        self.state = None       # (group, k, v, dk, dv) of the split sequence being processed

    def _ensure_workspace(self, fp):
        need = B.cf_attn_bwd_workspace_bytes(fp)
        if need > self._ws_bytes:
            self.workspace = torch.empty(need, dtype=torch.uint8, device=self.dev)
            self._ws_bytes = need

    def _open_group(self, g):
        sid = int(self.plan.group_seq_id[g])
        if sid < 0:
            return
        L = self.seq_len[sid]
        k = torch.full((L, self.Hkv, self.D), float("nan"), dtype=self.tdtype, device=self.dev)   # poisoned until written
        v = torch.full_like(k, float("nan"))
        dk = torch.zeros((L, self.Hkv, self.D), dtype=torch.float32, device=self.dev)
        dv = torch.zeros_like(dk)
        self.state = {"group": g, "k": k, "v": v, "dk": dk, "dv": dv, "rows": 0}

    def _close_group(self, g):
        if self.state is not None and self.state["group"] == g:
            self.host_state[g] = {"dk": self.state["dk"].cpu(), "dv": self.state["dv"].cpu()}
            self.state = None

    def _params(self, c, slot):
        """Forward parameters of chunk c with its activations in `slot`; the chunk's keys must be in place."""
        p = self.plan
        T, P = int(p.chunk_tokens[c]), int(p.chunk_prefix_len[c])
        cu_q, cu_k = self.cu[c]
        lse = slot.lse[:self.Hq * T].view(self.Hq, T)
        if self.state is not None and self.state["group"] == int(p.chunk_group[c]):
            k, v = self.state["k"][:P + T], self.state["v"][:P + T]
        else:
            k, v = self.kv[0][:T], self.kv[1][:T]
        return B.make_fwd_params(slot.q[:T], k, v, slot.o[:T], lse, cu_q, cu_k, self.scale, self.flags)

    def _forward(self, c, keep):
        p, h = self.plan, self.host[c]
        T, P = int(p.chunk_tokens[c]), int(p.chunk_prefix_len[c])
        g = int(p.chunk_group[c])
        if keep:
            free = [s for s in self.slots if s.chunk is None]
            if not free:
                raise RuntimeError(f"Algorithm 2 with K = {self.K} asked for more than K kept chunks")
            slot = free[0]
            slot.chunk = c
            self.peak_slots = max(self.peak_slots, sum(s.chunk is not None for s in self.slots))
        else:
            slot = self.scratch
        slot.q[:T].copy_(h["q"], non_blocking=True)
        if self.state is not None and self.state["group"] == g:
            if self.state["rows"] < P + T:                 # first forward of this chunk: its keys enter the state
                if self.state["rows"] != P:
                    raise RuntimeError("forward passes of a group must run in ascending order (section 4.2)")
                self.state["k"][P:P + T].copy_(h["k"], non_blocking=True)
                self.state["v"][P:P + T].copy_(h["v"], non_blocking=True)
                self.state["rows"] = P + T
        else:
            self.kv[0][:T].copy_(h["k"], non_blocking=True)
            self.kv[1][:T].copy_(h["v"], non_blocking=True)
        fp = self._params(c, slot)
        B.cf_attn_fwd(fp)
        self.n_forward += 1
        h["o"].copy_(slot.o[:T], non_blocking=True)          # what the next layer consumes
        h["lse"].copy_(slot.lse[:self.Hq * T].view(self.Hq, T), non_blocking=True)
        if not keep:
            slot.poison()                                    # discarded: nothing may read these activations again

    def _backward(self, c):
        p, h = self.plan, self.host[c]
        T, P = int(p.chunk_tokens[c]), int(p.chunk_prefix_len[c])
        g = int(p.chunk_group[c])
        held = [s for s in self.slots if s.chunk == c]
        if not held:
            raise RuntimeError(f"backward of chunk {c} without kept activations: a discarded chunk must run "
                               "forward again first (Algorithm 2)")
        slot = held[0]
        fp = self._params(c, slot)
        self._ensure_workspace(fp)
        self.d_o[:T].copy_(h["d_o"], non_blocking=True)
        if self.state is not None and self.state["group"] == g:
            dk, dv = self.state["dk"][:P + T], self.state["dv"][:P + T]
        else:
            self.dkv[:, :T].zero_()
            dk, dv = self.dkv[0][:T], self.dkv[1][:T]
        B.cf_attn_bwd(B.make_bwd_params(fp, self.d_o[:T], self.d_q[:T], dk, dv, self.workspace))
        self.n_backward += 1
        h["d_q"].copy_(self.d_q[:T], non_blocking=True)
        if "dk" in h:
            h["dk"].copy_(dk, non_blocking=True)
            h["dv"].copy_(dv, non_blocking=True)
        slot.poison()                                        # the slot is free again (stream order: after the copies)

    def run(self, ops=None):
        """Runs Algorithm 2's schedule for K (or the given op list, same format as Plan.schedule)."""
        p = self.plan
        ops = p.schedule(self.K) if ops is None else list(ops)
        self._allocate()
        current = None
        for op, c in ops:
            g = int(p.chunk_group[c])
            if g != current:
                if current is not None:
                    self._close_group(current)
                self._open_group(g)
                current = g
            if op == B.CF_OP_BWD:
                self._backward(c)
            else:
                self._forward(c, keep=op == B.CF_OP_FWD_KEEP)
        if current is not None:
            self._close_group(current)
        torch.cuda.synchronize()
        return self

    def device_bytes(self):
        """What the executor holds on the GPU by construction, by kind (bytes)."""
        slot = self.slots[0].bytes()
        row = self.Hkv * self.D
        longest = max([self.seq_len[int(s)] for s in self.plan.group_seq_id if int(s) >= 0], default=0)
        return {"activation_slots": self.K * slot, "scratch_slot": slot,
                "transient": sum(t.numel() * t.element_size() for t in (self.d_o, self.d_q, self.kv, self.dkv)),
                "state": longest * row * (2 * self.kv.element_size() + 2 * 4), "workspace": self._ws_bytes}

    # ------------------------------------------------------------------ results
    def results(self):
        """Per input sequence: o, lse, dq, dk, dv as fp64 numpy arrays (re-indexed through the plan)."""
        p, out = self.plan, {}
        f64 = lambda t: t.to(torch.float64).numpy()
        for c in range(p.n_chunks):
            h = self.host[c]
            cu = p.chunk_cu_seqlens(c)
            g = int(p.chunk_group[c])
            split = int(p.group_seq_id[g]) >= 0
            o, lse, dq = f64(h["o"]), f64(h["lse"]), f64(h["d_q"])
            for i, (sid, start, n) in enumerate(p.chunk_segments(c)):
                a, b = int(cu[i]), int(cu[i + 1])
                r = out.setdefault(sid, {})
                if split:
                    L = self.seq_len[sid]
                    if "o" not in r:
                        r.update(o=np.zeros((L, self.Hq, self.D)), lse=np.zeros((self.Hq, L)),
                                 dq=np.zeros((L, self.Hq, self.D)), dk=f64(self.host_state[g]["dk"]),
                                 dv=f64(self.host_state[g]["dv"]))
                    r["o"][start:start + n], r["dq"][start:start + n] = o[a:b], dq[a:b]
                    r["lse"][:, start:start + n] = lse[:, a:b]
                else:
                    r.update(o=o[a:b], lse=lse[:, a:b], dq=dq[a:b], dk=f64(h["dk"])[a:b], dv=f64(h["dv"])[a:b])
        return out
