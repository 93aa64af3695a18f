"""Pins for the fp64 attention oracle (CPU only).

Each check compares oracle/attention.c with something that is not itself: a dense-mask brute force
written here with central finite differences for the gradients, PyTorch's CPU scaled-dot-product
attention with autograd, closed forms, and the paper's equivalence claims (section 4: chunked
execution with accumulated gradients equals ordinary training; section 2.2: packing keeps
sequences independent; section 4.2: later chunks read the key/value state of earlier ones).
"""
import numpy as np
import pytest
import torch

from oracle import attention as A
from oracle import chunking as CK
from oracle.run_plan import run_plan, run_unsplit


def rand(rng, *shape):
    return rng.standard_normal(shape)


# ----------------------------------------------------------------------------- brute force
def dense_mask(cu_q, cu_k):
    """allowed[t, u]: query row t and key row u are in the same segment and the key's position in
    the sequence is not after the query's (query local i sits at position (Lk - Lq) + i)."""
    Tq, Tk = cu_q[-1], cu_k[-1]
    q_seg = np.zeros(Tq, int); q_pos = np.zeros(Tq, int)
    k_seg = np.zeros(Tk, int); k_pos = np.zeros(Tk, int)
    for g in range(len(cu_q) - 1):
        lq, lk = cu_q[g + 1] - cu_q[g], cu_k[g + 1] - cu_k[g]
        q_seg[cu_q[g]:cu_q[g + 1]] = g
        q_pos[cu_q[g]:cu_q[g + 1]] = (lk - lq) + np.arange(lq)
        k_seg[cu_k[g]:cu_k[g + 1]] = g
        k_pos[cu_k[g]:cu_k[g + 1]] = np.arange(lk)
    return (q_seg[:, None] == k_seg[None, :]) & (k_pos[None, :] <= q_pos[:, None])


def brute_fwd(q, k, v, mask, scale):
    Hq, Hkv = q.shape[1], k.shape[1]
    G = Hq // Hkv
    o = np.zeros_like(q); lse = np.zeros((Hq, q.shape[0]))
    for h in range(Hq):
        s = scale * q[:, h, :] @ k[:, h // G, :].T
        s = np.where(mask, s, -np.inf)
        e = np.exp(s)                     # tiny inputs: no range problem, softmax by definition
        z = e.sum(axis=1)
        o[:, h, :] = (e / z[:, None]) @ v[:, h // G, :]
        lse[h] = np.log(z)
    return o, lse


def fd_grads(q, k, v, d_o, mask, scale, eps=1e-5):
    """Central differences of l = <O, dO> with respect to every input element."""
    def loss(q_, k_, v_):
        return float((brute_fwd(q_, k_, v_, mask, scale)[0] * d_o).sum())
    grads = []
    for idx, x in enumerate((q, k, v)):
        g = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            args = [q.copy(), k.copy(), v.copy()]
            args[idx][i] += eps; lp = loss(*args)
            args[idx][i] -= 2 * eps; lm = loss(*args)
            g[i] = (lp - lm) / (2 * eps)
        grads.append(g)
    return grads


@pytest.mark.parametrize("cu_q,cu_k,Hq,Hkv", [
    ([0, 5], [0, 5], 1, 1),                      # one plain sequence
    ([0, 3, 4, 9], [0, 3, 4, 9], 2, 1),          # packed, incl. a length-1 sequence, GQA
    ([0, 4], [0, 11], 2, 2),                     # dependent chunk with 7 prefix keys
    ([0, 2, 6], [0, 2, 13], 4, 2),               # mixed: own-only segment and a prefixed one
])
def test_chunk_oracle_vs_bruteforce_and_finite_differences(cu_q, cu_k, Hq, Hkv):
    rng = np.random.default_rng(1)
    D, scale = 4, 0.37
    q, d_o = rand(rng, cu_q[-1], Hq, D), rand(rng, cu_q[-1], Hq, D)
    k, v = rand(rng, cu_k[-1], Hkv, D), rand(rng, cu_k[-1], Hkv, D)
    mask = dense_mask(cu_q, cu_k)
    o_ref, lse_ref = brute_fwd(q, k, v, mask, scale)
    o, lse = A.chunk_attn_fwd(q, k, v, cu_q, cu_k, scale)
    np.testing.assert_allclose(o, o_ref, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse, lse_ref, rtol=0, atol=1e-13)
    dq_fd, dk_fd, dv_fd = fd_grads(q, k, v, d_o, mask, scale)
    dk0, dv0 = rand(rng, *k.shape), rand(rng, *v.shape)      # non-zero start: must be added to
    dk, dv = dk0.copy(), dv0.copy()
    dq = A.chunk_attn_bwd(q, k, v, o, lse, d_o, cu_q, cu_k, scale, dk, dv)
    np.testing.assert_allclose(dq, dq_fd, rtol=0, atol=2e-9)
    np.testing.assert_allclose(dk - dk0, dk_fd, rtol=0, atol=2e-9)
    np.testing.assert_allclose(dv - dv0, dv_fd, rtol=0, atol=2e-9)


def test_seq_oracle_vs_bruteforce_and_finite_differences():
    rng = np.random.default_rng(2)
    L, Hq, Hkv, D, scale = 7, 4, 2, 3, 0.5
    q, d_o, k, v = rand(rng, L, Hq, D), rand(rng, L, Hq, D), rand(rng, L, Hkv, D), rand(rng, L, Hkv, D)
    mask = np.tril(np.ones((L, L), bool))
    o_ref, lse_ref = brute_fwd(q, k, v, mask, scale)
    o, lse = A.seq_attn_fwd(q, k, v, scale)
    np.testing.assert_allclose(o, o_ref, atol=1e-13, rtol=0)
    np.testing.assert_allclose(lse, lse_ref, atol=1e-13, rtol=0)
    dq, dk, dv = A.seq_attn_bwd(q, k, v, o, lse, d_o, scale)
    dq_fd, dk_fd, dv_fd = fd_grads(q, k, v, d_o, mask, scale)
    np.testing.assert_allclose(dq, dq_fd, atol=2e-9, rtol=0)
    np.testing.assert_allclose(dk, dk_fd, atol=2e-9, rtol=0)
    np.testing.assert_allclose(dv, dv_fd, atol=2e-9, rtol=0)


# ----------------------------------------------------------------------------- library routine
@pytest.mark.parametrize("Hq,Hkv", [(3, 3), (6, 2)])
def test_seq_oracle_vs_torch_sdpa_fp64(Hq, Hkv):
    """One sequence, one chunk: ordinary causal scaled-dot-product attention.  GQA must equal
    multi-head attention with each key/value head repeated (and its gradient summed)."""
    rng = np.random.default_rng(3)
    L, D = 61, 16
    scale = 1.0 / np.sqrt(D)
    q, d_o, k, v = rand(rng, L, Hq, D), rand(rng, L, Hq, D), rand(rng, L, Hkv, D), rand(rng, L, Hkv, D)
    tq = torch.tensor(q).permute(1, 0, 2).clone().requires_grad_()          # [H, L, D]
    tk = torch.tensor(k).permute(1, 0, 2).clone().requires_grad_()
    tv = torch.tensor(v).permute(1, 0, 2).clone().requires_grad_()
    G = Hq // Hkv
    to = torch.nn.functional.scaled_dot_product_attention(
        tq[None], tk.repeat_interleave(G, 0)[None], tv.repeat_interleave(G, 0)[None],
        is_causal=True, scale=scale)[0]
    to.backward(torch.tensor(d_o).permute(1, 0, 2))
    o, lse = A.seq_attn_fwd(q, k, v, scale)
    dq, dk, dv = A.seq_attn_bwd(q, k, v, o, lse, d_o, scale)
    np.testing.assert_allclose(o, to.detach().permute(1, 0, 2).numpy(), atol=1e-12, rtol=0)
    np.testing.assert_allclose(dq, tq.grad.permute(1, 0, 2).numpy(), atol=1e-12, rtol=0)
    np.testing.assert_allclose(dk, tk.grad.permute(1, 0, 2).numpy(), atol=1e-12, rtol=0)
    np.testing.assert_allclose(dv, tv.grad.permute(1, 0, 2).numpy(), atol=1e-12, rtol=0)
    # chunk form with Lk == Lq is the same thing
    o2, lse2 = A.chunk_attn_fwd(q, k, v, [0, L], [0, L], scale)
    np.testing.assert_allclose(o2, o, atol=1e-14, rtol=0)
    np.testing.assert_allclose(lse2, lse, atol=1e-14, rtol=0)


# ----------------------------------------------------------------------------- closed forms
def test_zero_queries_give_running_mean_and_log_position():
    """Q = 0: every visible key weighs the same, so O_i is the mean of v_0..v_pos and
    LSE_i = ln(pos + 1) with pos the position in the WHOLE sequence (prefix included)."""
    rng = np.random.default_rng(4)
    P, T, H, D = 9, 5, 2, 3
    k, v = rand(rng, P + T, H, D), rand(rng, P + T, H, D)
    q = np.zeros((T, H, D))
    o, lse = A.chunk_attn_fwd(q, k, v, [0, T], [0, P + T], 0.7)
    for i in range(T):
        np.testing.assert_allclose(o[i], v[:P + i + 1].mean(axis=0), atol=1e-14)
        np.testing.assert_allclose(lse[:, i], np.log(P + i + 1), atol=1e-14)


def test_constant_values_length_one_and_key_shift():
    rng = np.random.default_rng(5)
    L, H, D, s = 12, 2, 4, 0.3
    q, k = rand(rng, L, H, D), rand(rng, L, H, D)
    c = rand(rng, H, D)
    o, lse = A.seq_attn_fwd(q, k, np.broadcast_to(c, (L, H, D)).copy(), s)
    np.testing.assert_allclose(o, np.broadcast_to(c, (L, H, D)), atol=1e-14)   # V constant => O constant
    v = rand(rng, L, H, D)
    o1, _ = A.seq_attn_fwd(q, k, v, s)
    o2, _ = A.seq_attn_fwd(q, k + rand(rng, 1, H, D), v, s)                   # same shift on all keys
    np.testing.assert_allclose(o1, o2, atol=1e-13)
    # a sequence of one token: O = v, dV = dO, dQ = dK = 0
    q1, k1, v1, do1 = rand(rng, 1, H, D), rand(rng, 1, H, D), rand(rng, 1, H, D), rand(rng, 1, H, D)
    o, lse = A.seq_attn_fwd(q1, k1, v1, s)
    dq, dk, dv = A.seq_attn_bwd(q1, k1, v1, o, lse, do1, s)
    np.testing.assert_allclose(o, v1, atol=1e-15)
    np.testing.assert_allclose(dv, do1, atol=1e-15)
    assert np.abs(dq).max() < 1e-15 and np.abs(dk).max() < 1e-15


# ----------------------------------------------------------------------------- paper invariants
def make_seqs(rng, lens, Hq, Hkv, D):
    return {i: {"q": rand(rng, L, Hq, D), "k": rand(rng, L, Hkv, D), "v": rand(rng, L, Hkv, D),
                "d_o": rand(rng, L, Hq, D)} for i, L in enumerate(lens)}


@pytest.mark.parametrize("C", [16, 25, 64, 10 ** 9])
def test_chunked_equals_unsplit(C):
    """Split long sequences with carried key/value state, packed short ones, gradients summed
    along the state dependency: all must equal whole-sequence attention, for any chunk size
    (dividing, non-dividing, never splitting)."""
    rng = np.random.default_rng(6)
    lens = [5, 70, 16, 1, 33, 9, 12, 51]
    Hq, Hkv, D, scale = 4, 2, 8, 0.35
    seqs = make_seqs(rng, lens, Hq, Hkv, D)
    chunks, groups = CK.build_chunks(lens, C)
    got = run_plan(chunks, groups, seqs, scale)
    ref = run_unsplit(seqs, scale)
    for sid in seqs:
        for name in ("o", "lse", "dq", "dk", "dv"):
            np.testing.assert_allclose(got[sid][name], ref[sid][name], atol=1e-12, rtol=0,
                                       err_msg=f"seq {sid} {name} C={C}")


@pytest.mark.parametrize("C", [16, 25, 40])
def test_chunked_with_merged_tails_equals_unsplit(C):
    """The same equivalence when the last slice of a split sequence shares a chunk with short sequences
    (a chunk whose segments mix 'keys longer than queries' with plain ones)."""
    rng = np.random.default_rng(8)
    lens = [5, 70, 16, 1, 33, 9, 12, 51, 3]
    Hq, Hkv, D, scale = 4, 2, 8, 0.35
    seqs = make_seqs(rng, lens, Hq, Hkv, D)
    chunks, groups = CK.build_chunks(lens, C, merge_tails=True)
    assert any(len(c["segments"]) > 1 and c["prefix_len"] > 0 for c in chunks)      # the case is exercised
    got = run_plan(chunks, groups, seqs, scale)
    ref = run_unsplit(seqs, scale)
    for sid in seqs:
        for name in ("o", "lse", "dq", "dk", "dv"):
            np.testing.assert_allclose(got[sid][name], ref[sid][name], atol=1e-12, rtol=0,
                                       err_msg=f"seq {sid} {name} C={C}")


def test_packed_chunk_equals_sequences_run_alone():
    rng = np.random.default_rng(7)
    lens = [4, 9, 1, 6]
    Hq, Hkv, D, s = 2, 1, 5, 0.4
    seqs = make_seqs(rng, lens, Hq, Hkv, D)
    cu = np.concatenate([[0], np.cumsum(lens)])
    cat = lambda n: np.concatenate([seqs[i][n] for i in range(len(lens))])
    o, lse = A.chunk_attn_fwd(cat("q"), cat("k"), cat("v"), cu, cu, s)
    dk, dv = np.zeros_like(cat("k")), np.zeros_like(cat("v"))
    dq = A.chunk_attn_bwd(cat("q"), cat("k"), cat("v"), o, lse, cat("d_o"), cu, cu, s, dk, dv)
    for i, L in enumerate(lens):
        oi, lsei = A.seq_attn_fwd(seqs[i]["q"], seqs[i]["k"], seqs[i]["v"], s)
        dqi, dki, dvi = A.seq_attn_bwd(seqs[i]["q"], seqs[i]["k"], seqs[i]["v"], oi, lsei, seqs[i]["d_o"], s)
        sl = slice(cu[i], cu[i + 1])
        np.testing.assert_allclose(o[sl], oi, atol=1e-13)
        np.testing.assert_allclose(lse[:, sl], lsei, atol=1e-13)
        np.testing.assert_allclose(dq[sl], dqi, atol=1e-13)
        np.testing.assert_allclose(dk[sl], dki, atol=1e-13)
        np.testing.assert_allclose(dv[sl], dvi, atol=1e-13)


def test_rejects_segment_with_more_queries_than_keys():
    z = np.zeros((3, 1, 2))
    with pytest.raises(ValueError):
        A.chunk_attn_fwd(z, z[:2], z[:2], [0, 3], [0, 2], 1.0)
