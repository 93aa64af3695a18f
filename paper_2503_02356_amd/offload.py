"""Key/value state offload for a split sequence (the paper's section 6.3 names it as future work: its implementation
keeps the key/value tensors of ALL layers in GPU memory, so a 256K context costs more memory than a 32K one at the
same ChunkSize).

A split sequence of L tokens passes through n_layers attention layers, chunk by chunk (section 4.2): forward over
the chunks in ascending order, each chunk through the layers in ascending order; backward over the chunks in
descending order, each through the layers in descending order.  Every layer has its own key/value state
[L, Hkv, D] and fp32 gradient state of the same shape.  Between two visits of a layer all other layers run, so its
state can wait in pinned host memory: here the GPU holds `window` state slots, and the state of the layer a slot
serves next is prefetched on a copy stream while the current layer computes; after the attention call the rows
that changed go back to the host on a second copy stream (forward: the chunk's own key/value rows [P, P+T);
backward: gradient rows [0, P+T)).  window >= n_layers keeps every layer's state resident and copies no state.

Memory placement and stream order only: every arithmetic step runs inside cf_attn_fwd / cf_attn_bwd.  What a
model's other layers produce and consume on the GPU (a layer's Q, K, V projections and dO; its O, LSE and dQ) stays
on the GPU in both modes alike and is not counted as state.
"""
import ctypes as C

import numpy as np
import torch

from . import binding as B


class _StateSlot:
    def __init__(self, L, Hkv, D, dtype, dev):
        self.k = torch.empty((L, Hkv, D), dtype=dtype, device=dev)
        self.v = torch.empty_like(self.k)
        self.dk = torch.empty((L, Hkv, D), dtype=torch.float32, device=dev)
        self.dv = torch.empty_like(self.dk)
        self.loaded = torch.cuda.Event()       # the copy stream has brought in what the next op reads
        self.computed = torch.cuda.Event()     # the compute stream is done with the slot
        self.free = torch.cuda.Event()         # the write-back stream has taken what the op produced
        self.layer = None                      # resident mode: the layer whose state the slot holds for good

    def bytes(self):
        ts = (self.k, self.v, self.dk, self.dv)
        return sum(t.numel() * t.element_size() for t in ts)


class LayeredSequenceAttention:
    def __init__(self, seq_len, chunk_size, n_layers, n_q_heads, n_kv_heads, head_dim, window, dtype="bf16",
                 device="cuda:0"):
        self.L, self.C, self.n_layers = int(seq_len), int(chunk_size), int(n_layers)
        self.Hq, self.Hkv, self.D = n_q_heads, n_kv_heads, head_dim
        self.window = max(1, min(int(window), self.n_layers))
        self.offload = self.window < self.n_layers
        self.tdtype = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.dev = torch.device(device)
        self.scale = 1.0 / float(np.sqrt(head_dim))
        self.plan = B.cf_build_chunks([self.L], self.C)          # Algorithm 1: the slices of the one sequence
        self.chunks = [(int(self.plan.chunk_prefix_len[c]), int(self.plan.chunk_tokens[c])) for c in self.plan.group(0)]
        self.host, self.act = [], []
        self.h2d_bytes = self.d2h_bytes = 0

    def load(self, values):
        """values(layer) -> dict(q, k, v, d_o) of fp32 numpy arrays [L, H, D]."""
        dt, dev = self.tdtype, self.dev
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev).to(dt)
        for l in range(self.n_layers):
            v = values(l)
            a = {name: up(v[name]) for name in ("q", "k", "v", "d_o")}           # the layer's projections and dO
            a["o"] = torch.empty_like(a["q"])
            a["d_q"] = torch.empty_like(a["q"])
            a["lse"] = [torch.empty((self.Hq, T), dtype=torch.float32, device=dev) for _, T in self.chunks]
            self.act.append(a)
            # the layer's state as the host holds it: key/value rows arrive when a chunk's forward has produced them
            h = {"k_state": torch.full((self.L, self.Hkv, self.D), float("nan"), dtype=dt).pin_memory(),
                 "v_state": torch.full((self.L, self.Hkv, self.D), float("nan"), dtype=dt).pin_memory(),
                 "dk_state": torch.full((self.L, self.Hkv, self.D), float("nan"), dtype=torch.float32).pin_memory(),
                 "dv_state": torch.full((self.L, self.Hkv, self.D), float("nan"), dtype=torch.float32).pin_memory()}
            self.host.append(h)
        self.slots = [_StateSlot(self.L, self.Hkv, self.D, dt, dev) for _ in range(self.window)]
        self.copy_in, self.copy_out = torch.cuda.Stream(device=dev), torch.cuda.Stream(device=dev)
        self.written = [torch.cuda.Event() for _ in range(self.n_layers)]   # per layer: its state on the host is up to date
        self.cu = {}
        ws = 0
        for P, T in self.chunks:
            self.cu[(P, T)] = (torch.tensor([0, T], dtype=torch.int32, device=dev),
                               torch.tensor([0, P + T], dtype=torch.int32, device=dev))
        for m, (P, T) in enumerate(self.chunks):
            ws = max(ws, B.cf_attn_bwd_workspace_bytes(self._params(self.slots[0], 0, m)))
        self.workspace = torch.empty(ws, dtype=torch.uint8, device=dev)     # ops run one at a time on the compute stream
        if not self.offload:
            for l, s in enumerate(self.slots):
                s.layer = l
                s.k.fill_(float("nan"))
                s.v.fill_(float("nan"))
        return self

    def device_bytes(self):
        return sum(s.bytes() for s in self.slots) + self.workspace.numel()

    def _params(self, s, layer, m):
        P, T = self.chunks[m]
        a = self.act[layer]
        cu_q, cu_k = self.cu[(P, T)]
        return B.make_fwd_params(a["q"][P:P + T], s.k[:P + T], s.v[:P + T], a["o"][P:P + T], a["lse"][m], cu_q, cu_k,
                                 self.scale)

    def _copy(self, dst, src):
        dst.copy_(src, non_blocking=True)
        n = src.numel() * src.element_size()
        if dst.is_cuda and not src.is_cuda:
            self.h2d_bytes += n
        elif src.is_cuda and not dst.is_cuda:
            self.d2h_bytes += n

    def _slot(self, n_op, layer):
        return self.slots[layer if not self.offload else n_op % self.window]

    def _prefetch(self, n_op, layer, m, backward):
        """Copy stream: bring the rows the op reads into its slot, once the slot's previous user has been written back."""
        if not self.offload:
            return
        P, T = self.chunks[m]
        h, s = self.host[layer], self._slot(n_op, layer)
        with torch.cuda.stream(self.copy_in):
            self.copy_in.wait_event(s.free)
            self.copy_in.wait_event(self.written[layer])      # the layer's last write-back has reached the host
            rows = P + T if backward else P                    # backward: everything it reads; forward: the retained prefix
            self._copy(s.k[:rows], h["k_state"][:rows])
            self._copy(s.v[:rows], h["v_state"][:rows])
            # (the sequence's last chunk runs its backward first: no later chunk has added anything yet, so its
            # gradient state does not travel in -- _compute clears it on the device)
            if backward and m < len(self.chunks) - 1:
                self._copy(s.dk[:rows], h["dk_state"][:rows])
                self._copy(s.dv[:rows], h["dv_state"][:rows])
            s.loaded.record(self.copy_in)

    def _compute(self, n_op, layer, m, backward):
        P, T = self.chunks[m]
        a, s = self.act[layer], self._slot(n_op, layer)
        cur = torch.cuda.current_stream()
        if self.offload:
            cur.wait_event(s.loaded)
        if not backward:                                       # this chunk's own keys/values enter the state
            s.k[P:P + T].copy_(a["k"][P:P + T])
            s.v[P:P + T].copy_(a["v"][P:P + T])
        elif self.offload and m == len(self.chunks) - 1:       # first backward of the layer: gradients start at zero
            s.dk[:P + T].zero_()                               # (fill kernels on the compute stream: the copy
            s.dv[:P + T].zero_()                               # streams carry nothing but copies)
        fp = self._params(s, layer, m)
        handle = C.c_void_p(cur.cuda_stream)
        if backward:
            B.cf_attn_bwd(B.make_bwd_params(fp, a["d_o"][P:P + T], a["d_q"][P:P + T], s.dk[:P + T], s.dv[:P + T],
                                            self.workspace), handle)
        else:
            B.cf_attn_fwd(fp, handle)
        if self.offload:
            s.computed.record(cur)

    def _write_back(self, n_op, layer, m, backward):
        """Second copy stream: the rows the op changed go back to the host; then the slot is free."""
        if not self.offload:
            return
        P, T = self.chunks[m]
        h, s = self.host[layer], self._slot(n_op, layer)
        with torch.cuda.stream(self.copy_out):
            self.copy_out.wait_event(s.computed)
            if backward:
                self._copy(h["dk_state"][:P + T], s.dk[:P + T])
                self._copy(h["dv_state"][:P + T], s.dv[:P + T])
            else:
                self._copy(h["k_state"][P:P + T], s.k[P:P + T])
                self._copy(h["v_state"][P:P + T], s.v[P:P + T])
            s.free.record(self.copy_out)
            self.written[layer].record(self.copy_out)

    def run_step(self):
        """Forward over all chunks and layers, then backward; returns when everything is back on the host."""
        self.h2d_bytes = self.d2h_bytes = 0
        # (offloaded: the host's gradient state needs no clearing -- the last chunk's backward, the first to run,
        # writes all of its rows back)
        if not self.offload:
            for s in self.slots:
                s.dk.zero_()
                s.dv.zero_()
        torch.cuda.synchronize()
        ops = [(layer, m, False) for m in range(len(self.chunks)) for layer in range(self.n_layers)]          # ascending (section 4.2)
        ops += [(layer, m, True) for m in reversed(range(len(self.chunks))) for layer in reversed(range(self.n_layers))]
        # The prefetch of an op is submitted up to window - 1 ops ahead of its compute (the copy engines take their work
        # in submission order: a prefetch submitted after the previous op's write-back would wait behind it) -- but never
        # before the write-back of an earlier op on the same layer has been submitted: it reads what that one writes.
        ahead = self.window - 1 if self.offload else 0
        done = 0                                               # ops [0, done) have been computed and written back
        for i in range(len(ops)):
            while done < i and (i - done > ahead or any(ops[j][0] == ops[i][0] for j in range(done, i))):
                self._compute(done, *ops[done])
                self._write_back(done, *ops[done])
                done += 1
            self._prefetch(i, *ops[i])
        while done < len(ops):
            self._compute(done, *ops[done])
            self._write_back(done, *ops[done])
            done += 1
        n_op = len(ops)
        torch.cuda.synchronize()
        return n_op

    def results(self, layer):
        """o, lse, dq, dk, dv of one layer as fp64 numpy arrays, keyed like the plan runner's results."""
        a, h = self.act[layer], self.host[layer]
        f64 = lambda t: t.detach().to(torch.float64).cpu().numpy()
        if self.offload:
            dk, dv = h["dk_state"], h["dv_state"]
        else:
            dk, dv = self.slots[layer].dk, self.slots[layer].dv
        lse = torch.cat(a["lse"], dim=1)
        return {0: dict(o=f64(a["o"]), lse=f64(lse), dq=f64(a["d_q"]), dk=f64(dk), dv=f64(dv))}
