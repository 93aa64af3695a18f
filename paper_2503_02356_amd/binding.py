"""ctypes binding of libchunkflow.so: same names as the C ABI, argument marshalling only.

PyTorch appears here only as the owner of device memory and streams (data_ptr(), current stream).
There is no CPU fallback: if the library is missing or an entry point fails, the call raises.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libchunkflow.so")

CF_OK, CF_EINVAL, CF_EUNSUPPORTED, CF_ENOMEM, CF_EHIP = 0, -1, -2, -3, -4
CF_BF16, CF_FP32 = 0, 1
CF_FLAG_SCALAR_KERNELS = 1
CF_FLAG_DKV_SINGLE_WRITER = 2
CF_OP_FWD_KEEP, CF_OP_FWD_DISCARD, CF_OP_BWD = 0, 1, 2

CF_PLAN_MERGE_TAILS = 1

EXPORTS = ["cf_last_error", "cf_version", "cf_build_chunks", "cf_build_chunks_ex", "cf_attn_q_tiles", "cf_plan_free", "cf_plan_get",
           "cf_build_schedule", "cf_schedule_stats", "cf_attn_fwd", "cf_attn_bwd_workspace_bytes", "cf_attn_bwd", "cf_attn_fwd_batch", "cf_attn_bwd_batch",
           "cf_count_pairs", "cf_profile_next_call", "cf_attn_bwd_static", "cf_sim_1f1b", "cf_sim_1f1b_sequences"]


class CfError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"chunkflow error {code}: {msg}")
        self.code = code


class PlanView(C.Structure):
    _fields_ = [("n_chunks", C.c_int64), ("n_segments", C.c_int64), ("n_groups", C.c_int64),
                ("total_tokens", C.c_int64), ("chunk_size", C.c_int64),
                ("chunk_seg_ptr", C.POINTER(C.c_int64)), ("chunk_tokens", C.POINTER(C.c_int32)),
                ("chunk_prefix_len", C.POINTER(C.c_int64)), ("chunk_group", C.POINTER(C.c_int32)),
                ("chunk_idx_in_group", C.POINTER(C.c_int32)), ("seg_seq_id", C.POINTER(C.c_int64)),
                ("seg_seq_start", C.POINTER(C.c_int64)), ("seg_len", C.POINTER(C.c_int32)),
                ("cu_seqlens", C.POINTER(C.c_int32)), ("group_chunk_ptr", C.POINTER(C.c_int64)),
                ("group_chunks", C.POINTER(C.c_int64)), ("group_seq_id", C.POINTER(C.c_int64))]


class SchedOp(C.Structure):
    _fields_ = [("op", C.c_int32), ("reserved", C.c_int32), ("chunk", C.c_int64)]


class SchedStats(C.Structure):
    _fields_ = [("n_forward", C.c_int64), ("n_backward", C.c_int64), ("n_reforward", C.c_int64),
                ("peak_kept_chunks", C.c_int64), ("peak_kept_tokens", C.c_int64), ("state_tokens", C.c_int64)]


class PipelineStats(C.Structure):
    _fields_ = [("makespan", C.c_int64), ("busy_per_stage", C.c_int64), ("bubble_ticks", C.c_int64),
                ("total_ticks", C.c_int64), ("n_ops", C.c_int64), ("n_stages", C.c_int32), ("reserved", C.c_int32)]


class AttnFwdParams(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("flags", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("softmax_scale", C.c_float), ("n_tokens", C.c_int32),
                ("n_kv_tokens", C.c_int32), ("n_segments", C.c_int32),
                ("cu_seqlens_q", C.c_void_p), ("cu_seqlens_k", C.c_void_p),
                ("q", C.c_void_p), ("q_stride_tok", C.c_int64), ("q_stride_head", C.c_int64),
                ("k", C.c_void_p), ("v", C.c_void_p), ("kv_stride_tok", C.c_int64), ("kv_stride_head", C.c_int64),
                ("o", C.c_void_p), ("o_stride_tok", C.c_int64), ("o_stride_head", C.c_int64),
                ("lse", C.c_void_p), ("q_tiles", C.c_void_p), ("n_q_tiles", C.c_int32)]


class AttnBwdParams(C.Structure):
    _fields_ = [("f", AttnFwdParams),
                ("d_o", C.c_void_p), ("do_stride_tok", C.c_int64), ("do_stride_head", C.c_int64),
                ("d_q", C.c_void_p), ("dq_stride_tok", C.c_int64), ("dq_stride_head", C.c_int64),
                ("d_k", C.c_void_p), ("d_v", C.c_void_p), ("dkv_stride_tok", C.c_int64), ("dkv_stride_head", C.c_int64),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_int64)]


_lib = None


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                               "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        L.cf_last_error.restype = C.c_char_p
        L.cf_version.restype = C.c_int
        L.cf_build_chunks.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.POINTER(C.c_void_p)]
        L.cf_build_chunks_ex.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_uint32, C.POINTER(C.c_void_p)]
        L.cf_plan_free.argtypes = [C.c_void_p]
        L.cf_plan_free.restype = None
        L.cf_plan_get.argtypes = [C.c_void_p, C.POINTER(PlanView)]
        L.cf_build_schedule.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.POINTER(SchedOp)), C.POINTER(C.c_int64)]
        L.cf_attn_fwd.argtypes = [C.POINTER(AttnFwdParams), C.c_void_p]
        L.cf_attn_bwd_workspace_bytes.argtypes = [C.POINTER(AttnFwdParams)]
        L.cf_attn_bwd_workspace_bytes.restype = C.c_int64
        L.cf_attn_bwd.argtypes = [C.POINTER(AttnBwdParams), C.c_void_p]
        L.cf_sim_1f1b.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_uint32, C.POINTER(PipelineStats)]
        L.cf_sim_1f1b_sequences.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.POINTER(PipelineStats)]
        L.cf_attn_bwd_static.argtypes = [C.POINTER(AttnBwdParams), C.c_void_p]
        L.cf_attn_fwd_batch.argtypes = [C.POINTER(AttnFwdParams), C.c_int32, C.c_void_p]
        L.cf_attn_bwd_batch.argtypes = [C.POINTER(AttnBwdParams), C.c_int32, C.c_void_p]
        L.cf_schedule_stats.argtypes = [C.c_void_p, C.c_int32, C.POINTER(SchedStats)]
        L.cf_profile_next_call.argtypes = [C.c_void_p, C.c_void_p]
        L.cf_count_pairs.argtypes = [C.c_void_p, C.c_void_p, C.c_int32]
        L.cf_count_pairs.restype = C.c_int64
        L.cf_attn_q_tiles.restype = C.c_int64
        L.cf_attn_q_tiles.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int64]
        _lib = L
    return _lib


def _check(rc):
    if rc < 0:
        raise CfError(rc, lib().cf_last_error().decode())
    return rc


def cf_version():
    return lib().cf_version()


class Plan:
    """Owns a cf_plan; arrays are copied out as numpy so they outlive nothing they should not."""

    def __init__(self, handle):
        self._h = handle
        v = PlanView()
        _check(lib().cf_plan_get(self._h, C.byref(v)))
        n_c, n_s, n_g = v.n_chunks, v.n_segments, v.n_groups

        def arr(ptr, n, dt):
            return np.ctypeslib.as_array(ptr, shape=(n,)).astype(dt, copy=True) if n > 0 else np.zeros(0, dt)
        self.n_chunks, self.n_segments, self.n_groups = n_c, n_s, n_g
        self.total_tokens, self.chunk_size = v.total_tokens, v.chunk_size
        self.chunk_seg_ptr = arr(v.chunk_seg_ptr, n_c + 1, np.int64)
        self.chunk_tokens = arr(v.chunk_tokens, n_c, np.int32)
        self.chunk_prefix_len = arr(v.chunk_prefix_len, n_c, np.int64)
        self.chunk_group = arr(v.chunk_group, n_c, np.int32)
        self.chunk_idx_in_group = arr(v.chunk_idx_in_group, n_c, np.int32)
        self.seg_seq_id = arr(v.seg_seq_id, n_s, np.int64)
        self.seg_seq_start = arr(v.seg_seq_start, n_s, np.int64)
        self.seg_len = arr(v.seg_len, n_s, np.int32)
        self.cu_seqlens = arr(v.cu_seqlens, n_s + n_c, np.int32)
        self.group_chunk_ptr = arr(v.group_chunk_ptr, n_g + 1, np.int64)
        self.group_chunks = arr(v.group_chunks, n_c, np.int64)
        self.group_seq_id = arr(v.group_seq_id, n_g, np.int64)

    def chunk_cu_seqlens(self, c):
        a = int(self.chunk_seg_ptr[c]) + c
        return self.cu_seqlens[a:a + int(self.chunk_seg_ptr[c + 1] - self.chunk_seg_ptr[c]) + 1]

    def chunk_segments(self, c):
        a, b = int(self.chunk_seg_ptr[c]), int(self.chunk_seg_ptr[c + 1])
        return [(int(self.seg_seq_id[s]), int(self.seg_seq_start[s]), int(self.seg_len[s])) for s in range(a, b)]

    def group(self, g):
        return [int(x) for x in self.group_chunks[int(self.group_chunk_ptr[g]):int(self.group_chunk_ptr[g + 1])]]

    def schedule(self, K):
        ops, n = C.POINTER(SchedOp)(), C.c_int64()
        _check(lib().cf_build_schedule(self._h, int(K), C.byref(ops), C.byref(n)))
        return [(ops[i].op, ops[i].chunk) for i in range(n.value)]

    def schedule_stats(self, K):
        """cf_schedule_stats as a dict."""
        st = SchedStats()
        _check(lib().cf_schedule_stats(self._h, int(K), C.byref(st)))
        return {name: int(getattr(st, name)) for name, _ in SchedStats._fields_}

    def sim_1f1b(self, K, n_stages, flags=0):
        """cf_sim_1f1b as a dict."""
        st = PipelineStats()
        _check(lib().cf_sim_1f1b(self._h, int(K), int(n_stages), int(flags), C.byref(st)))
        return {name: int(getattr(st, name)) for name, _ in PipelineStats._fields_ if name != "reserved"}

    def close(self):
        if self._h:
            lib().cf_plan_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def cf_build_chunks(seq_lens, chunk_size):
    lens = np.ascontiguousarray(seq_lens, dtype=np.int64)
    h = C.c_void_p()
    _check(lib().cf_build_chunks(lens.ctypes.data_as(C.c_void_p), len(lens), int(chunk_size), C.byref(h)))
    return Plan(h)


def cf_build_chunks_ex(seq_lens, chunk_size, flags):
    lens = np.ascontiguousarray(seq_lens, dtype=np.int64)
    h = C.c_void_p()
    _check(lib().cf_build_chunks_ex(lens.ctypes.data_as(C.c_void_p), len(lens), int(chunk_size), int(flags), C.byref(h)))
    return Plan(h)


CF_SIM_PLAN_ORDER = 1


def cf_sim_1f1b_sequences(seq_lens, n_stages):
    lens = np.ascontiguousarray(seq_lens, dtype=np.int64)
    st = PipelineStats()
    _check(lib().cf_sim_1f1b_sequences(lens.ctypes.data_as(C.c_void_p), len(lens), int(n_stages), C.byref(st)))
    return {name: int(getattr(st, name)) for name, _ in PipelineStats._fields_ if name != "reserved"}


def cf_count_pairs(cu_q, cu_k):
    a = np.ascontiguousarray(cu_q, dtype=np.int32)
    b = np.ascontiguousarray(cu_k, dtype=np.int32)
    return _check(lib().cf_count_pairs(a.ctypes.data_as(C.c_void_p), b.ctypes.data_as(C.c_void_p), len(a) - 1))


def cf_profile_next_call(start_event, stop_event):
    """torch.cuda.Event pair (enable_timing=True) recorded around the next call's main kernel."""
    for e in (start_event, stop_event):
        if e is not None and not e.cuda_event:      # torch creates the hipEvent lazily: force it
            e.record()
    lib().cf_profile_next_call(C.c_void_p(start_event.cuda_event) if start_event is not None else None,
                               C.c_void_p(stop_event.cuda_event) if stop_event is not None else None)


def _dtype_code(t):
    import torch
    if t.dtype == torch.bfloat16:
        return CF_BF16
    if t.dtype == torch.float32:
        return CF_FP32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def cf_attn_q_tiles(cu_q, cu_k):
    """Host table of the chunk's 128-row query tiles, heaviest first: int32 array [n_tiles, 8] with the columns
    of cf_q_tile (q_begin, q_len, k_begin, k_len, tile, segment, 0, 0).  cu_q, cu_k: host int arrays."""
    a = np.ascontiguousarray(cu_q, dtype=np.int32)
    b = np.ascontiguousarray(cu_k, dtype=np.int32)
    n = _check(lib().cf_attn_q_tiles(a.ctypes.data_as(C.c_void_p), b.ctypes.data_as(C.c_void_p), len(a) - 1, None, 0))
    out = np.zeros((n, 8), dtype=np.int32)
    _check(lib().cf_attn_q_tiles(a.ctypes.data_as(C.c_void_p), b.ctypes.data_as(C.c_void_p), len(a) - 1,
                                 out.ctypes.data_as(C.c_void_p), n))
    return out


def make_fwd_params(q, k, v, o, lse, cu_q, cu_k, scale, flags=0, q_tiles=None):
    """q,o [T,Hq,D]; k,v [Tk,Hkv,D] (views with the same strides); lse [Hq,T] fp32 contiguous;
    cu_q, cu_k int32 device tensors [n_seg+1]; q_tiles: optional int32 device tensor [n_tiles, 8], the
    uploaded result of cf_attn_q_tiles for the same cu_seqlens."""
    T, Hq, D = q.shape
    Tk, Hkv, _ = k.shape
    assert q.is_cuda and q.stride(2) == 1 and k.stride(2) == 1 and v.stride() == k.stride() and o.stride(2) == 1
    assert lse.is_contiguous() and tuple(lse.shape) == (Hq, T)
    p = AttnFwdParams()
    p.dtype, p.flags = _dtype_code(q), int(flags)
    p.n_q_heads, p.n_kv_heads, p.head_dim = Hq, Hkv, D
    p.softmax_scale = float(scale)
    p.n_tokens, p.n_kv_tokens, p.n_segments = T, Tk, cu_q.numel() - 1
    p.cu_seqlens_q, p.cu_seqlens_k = cu_q.data_ptr(), cu_k.data_ptr()
    p.q, p.q_stride_tok, p.q_stride_head = q.data_ptr(), q.stride(0), q.stride(1)
    p.k, p.v, p.kv_stride_tok, p.kv_stride_head = k.data_ptr(), v.data_ptr(), k.stride(0), k.stride(1)
    p.o, p.o_stride_tok, p.o_stride_head = o.data_ptr(), o.stride(0), o.stride(1)
    p.lse = lse.data_ptr()
    if q_tiles is not None:
        assert q_tiles.is_cuda and q_tiles.is_contiguous() and q_tiles.element_size() == 4 and q_tiles.shape[1] == 8
        p.q_tiles, p.n_q_tiles = q_tiles.data_ptr(), q_tiles.shape[0]
    # The struct only carries raw addresses: keep the tensors alive as long as it lives, or the allocator may
    # hand their memory (e.g. a temporary cu_seqlens tensor) to someone else before the kernels have read it.
    p._keepalive = (q, k, v, o, lse, cu_q, cu_k, q_tiles)
    return p


def cf_attn_fwd(params, stream=None):
    _check(lib().cf_attn_fwd(C.byref(params), stream if stream is not None else _stream()))


def cf_attn_bwd_workspace_bytes(params):
    return _check(lib().cf_attn_bwd_workspace_bytes(C.byref(params)))


CF_STATIC_SCRATCH_BYTES = 16 << 20


def make_bwd_params(fwd_params, d_o, d_q, d_k, d_v, workspace):
    """workspace: uint8 device tensor, or None for cf_attn_bwd_static (which ignores the field)."""
    b = AttnBwdParams()
    b.f = fwd_params
    b.d_o, b.do_stride_tok, b.do_stride_head = d_o.data_ptr(), d_o.stride(0), d_o.stride(1)
    b.d_q, b.dq_stride_tok, b.dq_stride_head = d_q.data_ptr(), d_q.stride(0), d_q.stride(1)
    assert d_k.stride() == d_v.stride() and d_k.stride(2) == 1
    b.d_k, b.d_v, b.dkv_stride_tok, b.dkv_stride_head = d_k.data_ptr(), d_v.data_ptr(), d_k.stride(0), d_k.stride(1)
    if workspace is not None:
        b.workspace, b.workspace_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    b._keepalive = (fwd_params, d_o, d_q, d_k, d_v, workspace)      # see make_fwd_params
    return b


def params_array(params_list):
    """A contiguous ctypes array holding copies of the given parameter structs (kept alive with their tensors)."""
    if not params_list:
        return None
    arr = (type(params_list[0]) * len(params_list))(*params_list)
    arr._keepalive = tuple(params_list)
    return arr


def cf_attn_fwd_batch(params_arr, stream=None):
    n = len(params_arr) if params_arr is not None else 0
    _check(lib().cf_attn_fwd_batch(params_arr, n, stream if stream is not None else _stream()))


def cf_attn_bwd_batch(params_arr, stream=None):
    n = len(params_arr) if params_arr is not None else 0
    _check(lib().cf_attn_bwd_batch(params_arr, n, stream if stream is not None else _stream()))


def cf_attn_bwd(params, stream=None):
    _check(lib().cf_attn_bwd(C.byref(params), stream if stream is not None else _stream()))


def cf_attn_bwd_static(params, stream=None):
    _check(lib().cf_attn_bwd_static(C.byref(params), stream if stream is not None else _stream()))
