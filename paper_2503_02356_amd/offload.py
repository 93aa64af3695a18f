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

Memory placement and stream order only: every arithmetic step runs inside cf_attn_fwd / cf_attn_bwd.  The chunk's
activations (Q, O, LSE, dO, dQ) stand for what a model's other layers produce and consume; they live in pinned
host memory and cross for the op that needs them, in both modes alike.
"""
import ctypes as C

import numpy as np
import torch

from . import binding as B


class _StateSlot:
    def __init__(self, L, chunk, Hq, Hkv, D, dtype, dev):
        self.k = torch.empty((L, Hkv, D), dtype=dtype, device=dev)
        self.v = torch.empty_like(self.k)
        self.dk = torch.empty((L, Hkv, D), dtype=torch.float32, device=dev)
        self.dv = torch.empty_like(self.dk)
        self.q = torch.empty((chunk, Hq, D), dtype=dtype, device=dev)
        self.o = torch.empty_like(self.q)
        self.d_o = torch.empty_like(self.q)
        self.d_q = torch.empty_like(self.q)
        self.lse = torch.empty(Hq * chunk, dtype=torch.float32, device=dev)
        self.loaded = torch.cuda.Event()       # the copy stream has brought in what the next op reads
        self.computed = torch.cuda.Event()     # the compute stream is done with the slot
        self.free = torch.cuda.Event()         # the write-back stream has taken what the op produced
        self.layer = None                      # resident mode: the layer whose state the slot holds for good

    def bytes(self):
        ts = (self.k, self.v, self.dk, self.dv, self.q, self.o, self.d_o, self.d_q, self.lse)
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
        self.host = []
        self.h2d_bytes = self.d2h_bytes = 0

    def load(self, values):
        """values(layer) -> dict(q, k, v, d_o) of fp32 numpy arrays [L, H, D]; kept in pinned host memory."""
        dt = self.tdtype
        pin = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dt).pin_memory()
        for l in range(self.n_layers):
            v = values(l)
            h = {name: pin(v[name]) for name in ("q", "k", "v", "d_o")}
            h["o"] = torch.empty((self.L, self.Hq, self.D), dtype=dt).pin_memory()
            h["d_q"] = torch.empty_like(h["o"]).pin_memory()
            h["lse"] = torch.empty((self.Hq, self.L), dtype=torch.float32).pin_memory()
            # the layer's state as the host holds it: key/value rows arrive when a chunk's forward has produced them
            h["k_state"] = torch.full((self.L, self.Hkv, self.D), float("nan"), dtype=dt).pin_memory()
            h["v_state"] = torch.full((self.L, self.Hkv, self.D), float("nan"), dtype=dt).pin_memory()
            h["dk_state"] = torch.zeros((self.L, self.Hkv, self.D), dtype=torch.float32).pin_memory()
            h["dv_state"] = torch.zeros((self.L, self.Hkv, self.D), dtype=torch.float32).pin_memory()
            self.host.append(h)
        dev = self.dev
        self.slots = [_StateSlot(self.L, self.C, self.Hq, self.Hkv, self.D, dt, dev) for _ in range(self.window)]
        self.copy_in, self.copy_out = torch.cuda.Stream(device=dev), torch.cuda.Stream(device=dev)
        self.cu = {}
        ws = 0
        for P, T in self.chunks:
            self.cu[(P, T)] = (torch.tensor([0, T], dtype=torch.int32, device=dev),
                               torch.tensor([0, P + T], dtype=torch.int32, device=dev))
        s = self.slots[0]
        for P, T in self.chunks:
            fp = self._params(s, P, T)
            ws = max(ws, B.cf_attn_bwd_workspace_bytes(fp))
        self.workspace = torch.empty(ws, dtype=torch.uint8, device=dev)     # ops run one at a time on the compute stream
        if not self.offload:
            for l, s in enumerate(self.slots):
                s.layer = l
                s.k.fill_(float("nan"))
                s.v.fill_(float("nan"))
        return self

    def device_bytes(self):
        return sum(s.bytes() for s in self.slots) + self.workspace.numel()

    def _params(self, s, P, T):
        cu_q, cu_k = self.cu[(P, T)]
        return B.make_fwd_params(s.q[:T], s.k[:P + T], s.v[:P + T], s.o[:T], s.lse[:self.Hq * T].view(self.Hq, T),
                                 cu_q, cu_k, self.scale)

    def _copy(self, dst, src):
        dst.copy_(src, non_blocking=True)
        n = src.numel() * src.element_size()
        if dst.is_cuda:
            self.h2d_bytes += n
        else:
            self.d2h_bytes += n

    def _op(self, n_op, layer, P, T, backward):
        h = self.host[layer]
        s = self.slots[layer if not self.offload else n_op % self.window]
        cur = torch.cuda.current_stream()
        with torch.cuda.stream(self.copy_in):
            self.copy_in.wait_event(s.free)                    # the slot's last op has been written back
            if self.offload:
                if backward:
                    self._copy(s.k[:P + T], h["k_state"][:P + T])
                    self._copy(s.v[:P + T], h["v_state"][:P + T])
                    self._copy(s.dk[:P + T], h["dk_state"][:P + T])
                    self._copy(s.dv[:P + T], h["dv_state"][:P + T])
                else:
                    self._copy(s.k[:P], h["k_state"][:P])      # the retained prefix
                    self._copy(s.v[:P], h["v_state"][:P])
            if not backward:                                   # this chunk's own keys/values, as its projection makes them
                self._copy(s.k[P:P + T], h["k"][P:P + T])
                self._copy(s.v[P:P + T], h["v"][P:P + T])
            self._copy(s.q[:T], h["q"][P:P + T])
            if backward:
                self._copy(s.o[:T], h["o"][P:P + T])
                self._copy(s.lse[:self.Hq * T].view(self.Hq, T), h["lse"][:, P:P + T])
                self._copy(s.d_o[:T], h["d_o"][P:P + T])
            s.loaded.record(self.copy_in)
        cur.wait_event(s.loaded)
        fp = self._params(s, P, T)
        handle = C.c_void_p(cur.cuda_stream)
        if backward:
            B.cf_attn_bwd(B.make_bwd_params(fp, s.d_o[:T], s.d_q[:T], s.dk[:P + T], s.dv[:P + T], self.workspace), handle)
        else:
            B.cf_attn_fwd(fp, handle)
        s.computed.record(cur)
        with torch.cuda.stream(self.copy_out):
            self.copy_out.wait_event(s.computed)
            if backward:
                self._copy(h["d_q"][P:P + T], s.d_q[:T])
                if self.offload:
                    self._copy(h["dk_state"][:P + T], s.dk[:P + T])
                    self._copy(h["dv_state"][:P + T], s.dv[:P + T])
            else:
                self._copy(h["o"][P:P + T], s.o[:T])
                self._copy(h["lse"][:, P:P + T], s.lse[:self.Hq * T].view(self.Hq, T))
                if self.offload:
                    self._copy(h["k_state"][P:P + T], s.k[P:P + T])
                    self._copy(h["v_state"][P:P + T], s.v[P:P + T])
            s.free.record(self.copy_out)

    def run_step(self):
        """Forward over all chunks and layers, then backward; returns when everything is back on the host."""
        self.h2d_bytes = self.d2h_bytes = 0
        for h in self.host:
            h["dk_state"].zero_()
            h["dv_state"].zero_()
        if not self.offload:
            for s in self.slots:
                s.dk.zero_()
                s.dv.zero_()
        torch.cuda.synchronize()
        n_op = 0
        for P, T in self.chunks:                               # ascending (section 4.2)
            for layer in range(self.n_layers):
                self._op(n_op, layer, P, T, backward=False)
                n_op += 1
        for P, T in reversed(self.chunks):                     # descending
            for layer in reversed(range(self.n_layers)):
                self._op(n_op, layer, P, T, backward=True)
                n_op += 1
        torch.cuda.synchronize()
        if not self.offload:                                   # resident gradient states come back once, at the end
            for l, s in enumerate(self.slots):
                self.host[l]["dk_state"].copy_(s.dk)
                self.host[l]["dv_state"].copy_(s.dv)
            torch.cuda.synchronize()
        return n_op

    def results(self, layer):
        h = self.host[layer]
        f64 = lambda t: t.to(torch.float64).numpy()
        return {0: dict(o=f64(h["o"]), lse=f64(h["lse"]), dq=f64(h["d_q"]), dk=f64(h["dk_state"]), dv=f64(h["dv_state"]))}
