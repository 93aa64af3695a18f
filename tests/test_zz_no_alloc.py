"""cf_attn_bwd_static (the backward for callers that cannot allocate: its scratch is a static device buffer of
the library) against cf_attn_bwd with a caller-provided workspace, through the C ABI: two calls in a row, the
second on a smaller chunk, so that the buffer still holds the larger call's delta and work list."""
import numpy as np
import pytest
import torch

from paper_2503_02356_amd import binding as B
from tests import parity as P

pytestmark = pytest.mark.gpu


def _chunk(seed, cu_q, cu_k, Hq, Hkv, D, dtype):
    g = torch.Generator(device="cuda:0")
    g.manual_seed(seed)
    T, Tk = int(cu_q[-1]), int(cu_k[-1])
    rnd = lambda *s: torch.randn(*s, generator=g, device="cuda:0").to(dtype)
    q, d_o, k, v = rnd(T, Hq, D), rnd(T, Hq, D), rnd(Tk, Hkv, D), rnd(Tk, Hkv, D)
    o = torch.empty_like(q)
    lse = torch.empty(Hq, T, device="cuda:0", dtype=torch.float32)
    dev = lambda a: torch.tensor(a, dtype=torch.int32, device="cuda:0")
    fp = B.make_fwd_params(q, k, v, o, lse, dev(cu_q), dev(cu_k), 1 / np.sqrt(D))
    B.cf_attn_fwd(fp)
    return fp, d_o, T, Tk


def _both(fp, d_o, T, Tk, Hq, Hkv, D, dtype):
    """-> (dq, dk, dv) of cf_attn_bwd with a workspace, and of cf_attn_bwd_static, same non-zero dK/dV start."""
    start = torch.randn(2, Tk, Hkv, D, device="cuda:0") * 0.5
    res = []
    for static in (False, True):
        dq = torch.full((T, Hq, D), 3.0, device="cuda:0", dtype=dtype)
        dkv = start.clone()
        if static:
            B.cf_attn_bwd_static(B.make_bwd_params(fp, d_o, dq, dkv[0], dkv[1], None))
        else:
            ws = torch.empty(B.cf_attn_bwd_workspace_bytes(fp), dtype=torch.uint8, device="cuda:0")
            B.cf_attn_bwd(B.make_bwd_params(fp, d_o, dq, dkv[0], dkv[1], ws))
        torch.cuda.synchronize()
        res.append((dq.double().cpu().numpy(), (dkv[0] - start[0]).double().cpu().numpy(),
                    (dkv[1] - start[1]).double().cpu().numpy()))
    return res


@pytest.mark.parametrize("dtype,D", [(torch.bfloat16, 128), (torch.float32, 64)])
def test_static_scratch_backward_matches_workspace_backward(dtype, D):
    Hq, Hkv = 8, 2
    name = "bf16" if dtype == torch.bfloat16 else "fp32"
    # first a larger chunk: short documents plus a slice behind a 1500-token prefix; then a smaller one
    shapes = [([0, 300, 301, 700, 1300], [0, 300, 301, 700, 2800]), ([0, 90, 250], [0, 90, 250])]
    for n, (cu_q, cu_k) in enumerate(shapes):
        fp, d_o, T, Tk = _chunk(40 + n, cu_q, cu_k, Hq, Hkv, D, dtype)
        (dq_a, dk_a, dv_a), (dq_b, dk_b, dv_b) = _both(fp, d_o, T, Tk, Hq, Hkv, D, dtype)
        assert np.array_equal(dq_a, dq_b), f"call {n}: dQ differs"          # single writer per element
        got = {0: dict(o=dq_b, lse=dq_b, dq=dq_b, dk=dk_b, dv=dv_b)}
        ref = {0: dict(o=dq_a, lse=dq_a, dq=dq_a, dk=dk_a, dv=dv_a)}
        errs = P.check(got, ref, name, f"call {n}")
        # (the query heads of a group meet in dK/dV through fp32 atomics: equal up to the order of the additions)
        assert errs["dk"][1] < 1e-5 and errs["dv"][1] < 1e-5, errs
        print(f"{name} call {n}: T={T} Tk={Tk}", {k: errs[k] for k in ("dq", "dk", "dv")}, flush=True)
