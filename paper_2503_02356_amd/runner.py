"""Executes a chunk plan on one GPU: the StateStore and the launch order of paper section 4.2.

Memory placement only -- every arithmetic step runs inside cf_attn_fwd / cf_attn_bwd.
Per long sequence one key/value state buffer [L,Hkv,D] and one fp32 gradient state of the same
shape stay resident; a dependent chunk's call passes their base pointers with n_kv_tokens = P+T,
so the prefix and the chunk's own rows are one contiguous range.  Packed chunks own their K/V.
"""
import numpy as np
import torch

from . import binding as B


def schedule_memory(plan, K, n_q_heads, n_kv_heads, head_dim, elem_bytes=2):
    """Bytes the attention path holds under Algorithm 2 with K kept chunks (section 4.2: memory is
    governed by K * ChunkSize, plus the key/value state of the sequence being processed).
      kept_activation_bytes: Q, O (elem_bytes each) and LSE (fp32) of the kept chunks at the peak
      state_bytes          : K, V (elem_bytes) and fp32 dK, dV of the longest split sequence
    Only counts from cf_schedule_stats are used; nothing is allocated."""
    st = plan.schedule_stats(K)
    per_token = n_q_heads * (2 * head_dim * elem_bytes + 4)
    per_state_token = n_kv_heads * head_dim * (2 * elem_bytes + 2 * 4)
    return dict(st, kept_activation_bytes=st["peak_kept_tokens"] * per_token,
                state_bytes=st["state_tokens"] * per_state_token)


class ChunkAttention:
    def __init__(self, plan, n_q_heads, n_kv_heads, head_dim, dtype, scale=None, device="cuda:0", flags=0,
                 n_streams=1, fused_launch=False, only_groups=None, tile_tables=True):
        """n_streams > 1: dependency groups are dealt over that many HIP streams (default priority), so that
        the last, partly filled wave of workgroups of one chunk's kernel overlaps with the next group's
        kernels.  The chunks of one group stay on one stream, in the order of section 4.2."""
        self.plan, self.Hq, self.Hkv, self.D = plan, n_q_heads, n_kv_heads, head_dim
        self.n_streams = max(1, int(n_streams))
        # fused_launch: run_forward / run_backward hand the whole plan to cf_attn_fwd_batch / cf_attn_bwd_batch
        # (one workspace per chunk); otherwise one cf_attn_fwd / cf_attn_bwd call per chunk.
        self.fused_launch = bool(fused_launch)
        # tile_tables: give every chunk's calls the table of cf_attn_q_tiles (built on the host when the plan is
        # placed: it only depends on the chunk's cu_seqlens), so that the kernels start their heaviest tiles first
        self.tile_tables = bool(tile_tables)
        self.tdtype = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.scale = float(scale) if scale is not None else 1.0 / float(np.sqrt(head_dim))
        self.dev, self.flags = torch.device(device), flags
        # only_groups: place and run just these dependency groups of the plan (a batch too large for one GPU's
        # memory is then run group by group, or sampled); the other chunks' entries stay None.
        self.only_groups = None if only_groups is None else set(int(g) for g in only_groups)
        self.chunks = []          # per chunk: dict of device tensors and params
        self.state = {}           # group id -> dict(k, v, dk, dv) for long sequences

    # ------------------------------------------------------------------ data placement
    def load(self, values):
        """values(seq_id, L) -> dict(q,k,v,d_o) of fp32 numpy arrays or torch tensors [L,H,D] (already
        representable in the compute dtype)."""
        p, dev, dt = self.plan, self.dev, self.tdtype
        up = lambda a: (a if torch.is_tensor(a) else torch.from_numpy(np.ascontiguousarray(a))).to(dev).to(dt)
        cache = {}

        def get(sid, L):
            if sid not in cache:
                cache.clear()     # segments of one sequence are consecutive in the plan; keep one
                cache[sid] = values(sid, L)
            return cache[sid]
        seq_len = {}
        for s in range(p.n_segments):
            sid = int(p.seg_seq_id[s])
            seq_len[sid] = max(seq_len.get(sid, 0), int(p.seg_seq_start[s]) + int(p.seg_len[s]))
        ws_bytes = 0
        # All fp32 dK/dV buffers (per long sequence, per packed chunk) are slices of ONE allocation, so that zeroing
        # the gradients of a step is one fill.
        row = self.Hkv * self.D
        # (every key row of the batch appears in exactly one buffer: a split sequence's rows in its state, a
        # short sequence's in its chunk)
        placed = lambda c: self.only_groups is None or int(p.chunk_group[c]) in self.only_groups
        arena_rows = sum(int(p.chunk_tokens[c]) for c in range(p.n_chunks) if placed(c))
        self.grad_arena = torch.zeros(2 * arena_rows * row, dtype=torch.float32, device=dev)
        self._grad_used = 0

        def grad_pair(n_rows):
            a = self._grad_used
            self._grad_used += 2 * n_rows * row
            dk = self.grad_arena[a:a + n_rows * row].view(n_rows, self.Hkv, self.D)
            dv = self.grad_arena[a + n_rows * row:a + 2 * n_rows * row].view(n_rows, self.Hkv, self.D)
            return dk, dv
        def group_state(g):
            """Key/value state and its fp32 gradients of the split sequence of group g, created at the group's
            first chunk.  When the group's last chunk also holds other sequences (a merged tail), the state is a
            slice of that chunk's key/value buffer, so that the chunk's keys are one contiguous array."""
            if g in self.state:
                return self.state[g]
            sid = int(p.group_seq_id[g])
            L = seq_len[sid]
            vals = get(sid, L)
            last_segs = p.chunk_segments(int(p.group(g)[-1]))
            if len(last_segs) == 1:
                gdk, gdv = grad_pair(L)
                st = {"k": up(vals["k"]), "v": up(vals["v"]), "dk": gdk, "dv": gdv}
            else:
                cu_k = np.concatenate([[0], np.cumsum([start + n for (_, start, n) in last_segs])]).astype(np.int32)
                rows = int(cu_k[-1])
                kbuf = torch.empty((rows, self.Hkv, self.D), dtype=dt, device=dev)
                vbuf = torch.empty_like(kbuf)
                gdk, gdv = grad_pair(rows)
                a = int(cu_k[[s[0] for s in last_segs].index(sid)])
                kbuf[a:a + L].copy_(up(vals["k"]))
                vbuf[a:a + L].copy_(up(vals["v"]))
                st = {"k": kbuf[a:a + L], "v": vbuf[a:a + L], "dk": gdk[a:a + L], "dv": gdv[a:a + L],
                      "merged": {"k": kbuf, "v": vbuf, "dk": gdk, "dv": gdv, "cu_k": cu_k}}
            self.state[g] = st
            return st

        for c in range(p.n_chunks):
            segs = p.chunk_segments(c)
            T, P = int(p.chunk_tokens[c]), int(p.chunk_prefix_len[c])
            g = int(p.chunk_group[c])
            if not placed(c):
                self.chunks.append(None)
                continue
            dependent = int(p.group_seq_id[g]) >= 0
            merged = dependent and len(segs) > 1
            ch = {"T": T, "P": P, "dependent": dependent, "merged": merged, "segs": segs, "group": g}
            ch["q"] = torch.empty((T, self.Hq, self.D), dtype=dt, device=dev)
            ch["d_o"] = torch.empty_like(ch["q"])
            ch["o"] = torch.empty_like(ch["q"])
            ch["d_q"] = torch.empty_like(ch["q"])
            ch["lse"] = torch.empty((self.Hq, T), dtype=torch.float32, device=dev)
            cu = p.chunk_cu_seqlens(c)
            ch["cu_q_host"] = cu.copy()
            ch["cu_q"] = torch.from_numpy(cu.copy()).to(dev)
            if dependent and not merged:
                sid, start, n = segs[0]
                L = seq_len[sid]
                st = group_state(g)
                vals = get(sid, L)
                ch["k"], ch["v"] = st["k"][:P + T], st["v"][:P + T]
                ch["dk"], ch["dv"] = st["dk"][:P + T], st["dv"][:P + T]
                ch["q"].copy_(up(vals["q"][start:start + n]))
                ch["d_o"].copy_(up(vals["d_o"][start:start + n]))
                ch["cu_k_host"] = np.array([0, P + T], dtype=np.int32)
            elif merged:
                # short sequences plus the last slice of the group's split sequence, whose keys are its whole state
                M = group_state(g)["merged"]
                ch["k"], ch["v"], ch["dk"], ch["dv"] = M["k"], M["v"], M["dk"], M["dv"]
                ch["cu_k_host"] = M["cu_k"].copy()
                for i, (sid, start, n) in enumerate(segs):
                    vals = get(sid, seq_len[sid])
                    a, b = int(cu[i]), int(cu[i + 1])
                    ch["q"][a:b].copy_(up(vals["q"][start:start + n]))
                    ch["d_o"][a:b].copy_(up(vals["d_o"][start:start + n]))
                    if start == 0:           # (the state rows were filled when the group was first met)
                        ka = int(M["cu_k"][i])
                        ch["k"][ka:ka + n].copy_(up(vals["k"]))
                        ch["v"][ka:ka + n].copy_(up(vals["v"]))
            else:
                ch["k"] = torch.empty((T, self.Hkv, self.D), dtype=dt, device=dev)
                ch["v"] = torch.empty_like(ch["k"])
                ch["dk"], ch["dv"] = grad_pair(T)
                for i, (sid, start, n) in enumerate(segs):
                    vals = get(sid, n)
                    a, b = int(cu[i]), int(cu[i + 1])
                    ch["q"][a:b].copy_(up(vals["q"]))
                    ch["d_o"][a:b].copy_(up(vals["d_o"]))
                    ch["k"][a:b].copy_(up(vals["k"]))
                    ch["v"][a:b].copy_(up(vals["v"]))
                ch["cu_k_host"] = cu.copy()
            ch["cu_k"] = torch.from_numpy(ch["cu_k_host"].copy()).to(dev)
            ch["pairs"] = B.cf_count_pairs(ch["cu_q_host"], ch["cu_k_host"])
            if self.tile_tables:
                ch["q_tiles"] = torch.from_numpy(B.cf_attn_q_tiles(ch["cu_q_host"], ch["cu_k_host"])).to(dev)
            ch["fwd"] = B.make_fwd_params(ch["q"], ch["k"], ch["v"], ch["o"], ch["lse"], ch["cu_q"], ch["cu_k"],
                                          self.scale, self.flags, q_tiles=ch.get("q_tiles"))
            ws_bytes = max(ws_bytes, B.cf_attn_bwd_workspace_bytes(ch["fwd"]))
            self.chunks.append(ch)
        # one backward workspace per stream: calls on different streams overlap
        self.workspaces = [torch.empty(ws_bytes, dtype=torch.uint8, device=dev) for _ in range(self.n_streams)]
        self.streams = [torch.cuda.Stream(device=dev) for _ in range(self.n_streams)] if self.n_streams > 1 else []
        # groups go, in plan order, to the stream with the least work so far (work = unmasked pairs)
        load, lane_of = [0] * self.n_streams, {}
        placed_chunks = [ch for ch in self.chunks if ch is not None]
        for ch in placed_chunks:
            if ch["group"] not in lane_of:
                lane_of[ch["group"]] = load.index(min(load))
            load[lane_of[ch["group"]]] += ch["pairs"]
        for ch in placed_chunks:
            ch["lane"] = lane_of[ch["group"]]
            if self.fused_launch:       # the chunks of a fused call are in flight together: a workspace each
                need = B.cf_attn_bwd_workspace_bytes(ch["fwd"])
                ch["workspace"] = torch.empty(need, dtype=torch.uint8, device=dev)
            ch["bwd"] = B.make_bwd_params(ch["fwd"], ch["d_o"], ch["d_q"], ch["dk"], ch["dv"],
                                          ch.get("workspace", self.workspaces[ch["lane"]]))
        if self.fused_launch:
            self.fwd_batch = B.params_array([self.chunks[c]["fwd"] for c in self.forward_order()])
            self.bwd_batch = B.params_array([self.chunks[c]["bwd"] for c in self.backward_order()])
        self.total_pairs = sum(ch["pairs"] for ch in placed_chunks)
        return self

    # ------------------------------------------------------------------ launches
    def zero_grads(self):
        self.grad_arena.zero_()

    def groups(self):
        return [g for g in range(self.plan.n_groups) if self.only_groups is None or g in self.only_groups]

    def forward_order(self):
        return [c for g in self.groups() for c in self.plan.group(g)]

    def backward_order(self):
        return [c for g in self.groups() for c in reversed(self.plan.group(g))]

    def _launch(self, ops):
        """ops: iterable of (is_backward, chunk id) in issue order.  One stream: plain launches on the current
        stream.  Several: every side stream first waits for what the current stream has queued, and the current
        stream waits for all of them at the end, so callers see ordinary stream semantics."""
        if not self.streams:
            for bwd, c in ops:
                (B.cf_attn_bwd if bwd else B.cf_attn_fwd)(self.chunks[c]["bwd" if bwd else "fwd"])
            return
        cur = torch.cuda.current_stream()
        start = torch.cuda.Event()
        start.record(cur)
        for st in self.streams:
            st.wait_event(start)
        for bwd, c in ops:
            ch = self.chunks[c]
            handle = B.C.c_void_p(self.streams[ch["lane"]].cuda_stream)
            (B.cf_attn_bwd if bwd else B.cf_attn_fwd)(ch["bwd" if bwd else "fwd"], handle)
        for st in self.streams:
            done = torch.cuda.Event()
            done.record(st)
            cur.wait_event(done)

    def run_forward(self, fused=None):
        """fused: None = as constructed; True needs fused_launch=True at construction."""
        if self.fused_launch if fused is None else fused:
            B.cf_attn_fwd_batch(self.fwd_batch)
        else:
            self._launch((False, c) for c in self.forward_order())      # ascending inside each group

    def run_backward(self, fused=None):
        if self.fused_launch if fused is None else fused:
            B.cf_attn_bwd_batch(self.bwd_batch)
        else:
            self._launch((True, c) for c in self.backward_order())      # descending inside each group

    def run_schedule(self, K):
        """Algorithm 2 with K kept chunks: chunks marked FWD_DISCARD run forward (their K/V state is
        what later chunks need) and run forward again right before their backward."""
        self._launch((op == B.CF_OP_BWD, c) for op, c in self.plan.schedule(K) if self.chunks[c] is not None)

    def capture_step(self, K=None):
        """One whole step (zeroing of the gradients, forward, backward; Algorithm 2 with K kept chunks when K is
        given) recorded into a HIP graph and returned: `graph.replay()` then re-issues it with one call.  The
        entry points suit capture as they are: they only enqueue kernels on the stream they are given -- no
        allocation, no synchronisation, no memset node (the gradients are cleared by a fill kernel).  Single
        stream only."""
        assert not self.streams, "capture_step records the single-stream launch order"
        step = (lambda: self.run_schedule(K)) if K is not None else (lambda: (self.run_forward(), self.run_backward()))
        self.zero_grads()
        step()                                   # every lazy initialisation happens outside the capture
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.zero_grads()
            step()
        return graph

    # ------------------------------------------------------------------ results
    def results(self):
        """Per input sequence: o, lse, dq, dk, dv as fp64 numpy arrays (re-indexed through the plan)."""
        torch.cuda.synchronize()
        out = {}
        f64 = lambda t: t.detach().to(torch.float64).cpu().numpy()
        split = {int(self.plan.group_seq_id[g]): g for g in self.state}     # split sequence -> its group
        for ch in self.chunks:
            if ch is None:
                continue
            o, lse, dq = f64(ch["o"]), f64(ch["lse"]), f64(ch["d_q"])
            dk = dv = None
            if not ch["dependent"] or ch["merged"]:
                dk, dv = f64(ch["dk"]), f64(ch["dv"])
            cu, cu_k = ch["cu_q_host"], ch["cu_k_host"]
            for i, (sid, start, n) in enumerate(ch["segs"]):
                a, b = int(cu[i]), int(cu[i + 1])
                r = out.setdefault(sid, {})
                if sid in split:
                    st = self.state[split[sid]]
                    L = st["k"].shape[0]
                    if "o" not in r:
                        r.update(o=np.zeros((L, self.Hq, self.D)), lse=np.zeros((self.Hq, L)),
                                 dq=np.zeros((L, self.Hq, self.D)), dk=f64(st["dk"]), dv=f64(st["dv"]))
                    r["o"][start:start + n], r["dq"][start:start + n] = o[a:b], dq[a:b]
                    r["lse"][:, start:start + n] = lse[:, a:b]
                else:
                    ka = int(cu_k[i])
                    r.update(o=o[a:b], lse=lse[:, a:b], dq=dq[a:b], dk=dk[ka:ka + n], dv=dv[ka:ka + n])
        return out
