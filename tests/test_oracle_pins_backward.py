"""Pins of the oracle's SSA gradient (the derivative of Eq. 4 that the sparse mid-training of the
Architecture section's Training paragraph needs), CPU only.

Pinned by: reverse-mode differentiation of a library attention routine under a mask written with
Python sets from the verbal definition; central finite differences of the oracle's own forward
(independent of any backward formula); the closed form for Q = 0; and the identity that the score
gradients of a row sum to zero, seen through shift invariance of the keys.
"""
import numpy as np
import pytest
import torch

import oracle


def _rand(shape, seed, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(shape, generator=g, dtype=torch.float32) * scale)


def _set_live(i, ns, win, block):
    """Live set from the verbal definition (token-granular when block is None)."""
    if block is None:
        return {j for j in range(i + 1) if j < ns or j > i - win}
    qb = i // block
    return {j for j in range(i + 1) if j // block < ns or j // block > qb - win}


def _autograd(q, k, v, dout, ns, win, block, scale, alias_dv=None):
    """Gradients from torch autograd through scaled_dot_product_attention (fp64) under a set-built mask."""
    B, S, Hq, _ = q.shape
    Hkv = k.shape[2]
    mask = torch.zeros(S, S, dtype=torch.bool)
    for i in range(S):
        for j in _set_live(i, ns, win, block):
            mask[i, j] = True
    qd = q.double().clone().requires_grad_(True)
    kd = k.double().clone().requires_grad_(True)
    if alias_dv is None:
        vd = v.double().clone().requires_grad_(True)
        v_used = vd
    else:
        vd = None
        v_used = kd[..., :alias_dv]
    G = Hq // Hkv
    o = torch.nn.functional.scaled_dot_product_attention(
        qd.permute(0, 2, 1, 3), kd.permute(0, 2, 1, 3).repeat_interleave(G, dim=1),
        v_used.permute(0, 2, 1, 3).repeat_interleave(G, dim=1), attn_mask=mask, scale=scale)
    (o.permute(0, 2, 1, 3) * dout.double()).sum().backward()
    return qd.grad.numpy(), kd.grad.numpy(), None if vd is None else vd.grad.numpy()


@pytest.mark.parametrize("B,Hq,Hkv,S,d,dv,ns,win,block", [
    (1, 1, 1, 40, 8, 6, 3, 7, None),
    (2, 4, 2, 33, 8, 5, 0, 5, None),
    (1, 2, 1, 50, 6, 6, 2, 100, None),      # window covers everything: causal attention
    (1, 4, 1, 45, 8, 6, 1, 2, 4),           # block-granular
    (1, 2, 2, 37, 4, 3, 0, 1, 5),
    (1, 3, 1, 29, 5, 4, 2, 1, 1),
])
def test_gradients_match_library_autograd_under_set_built_mask(B, Hq, Hkv, S, d, dv, ns, win, block):
    q, k, v, dout = _rand((B, S, Hq, d), 1), _rand((B, S, Hkv, d), 2), _rand((B, S, Hkv, dv), 3), _rand((B, S, Hq, dv), 4)
    scale = 0.41
    dq, dk, dvv = oracle.ssa_backward(q, k, v, dout, n_sink=ns, window=win, scale=scale, block=block)
    rq, rk, rv = _autograd(q, k, v, dout, ns, win, block, scale)
    np.testing.assert_allclose(dq, rq, atol=1e-11)
    np.testing.assert_allclose(dk, rk, atol=1e-11)
    np.testing.assert_allclose(dvv, rv, atol=1e-11)


@pytest.mark.parametrize("ns,win,block", [(2, 6, None), (1, 2, 4)])
def test_aliased_values_gradient_of_the_shared_tensor(ns, win, block):
    """Values = first d_v columns of the keys: autograd differentiates the one tensor; the oracle's
    separate dk and dv must add up to it."""
    B, S, Hq, d, dv, scale = 1, 36, 4, 10, 6, 0.3
    q, k, dout = _rand((B, S, Hq, d), 11), _rand((B, S, 1, d), 12), _rand((B, S, Hq, dv), 13)
    dq, dk, dvv = oracle.ssa_backward(q, k, ("alias", dv), dout, n_sink=ns, window=win, scale=scale, block=block)
    rq, rk, _ = _autograd(q, k, None, dout, ns, win, block, scale, alias_dv=dv)
    total = dk.copy()
    total[..., :dv] += dvv
    np.testing.assert_allclose(dq, rq, atol=1e-11)
    np.testing.assert_allclose(total, rk, atol=1e-11)


def _forward_loss(q, k, v, dout, ns, win, block, scale):
    B, S, Hq, _ = q.shape
    b, i, h = np.meshgrid(np.arange(B), np.arange(S), np.arange(Hq), indexing="ij")
    rb, ri, rh = b.ravel(), i.ravel(), h.ravel()
    qr = q[torch.as_tensor(rb), torch.as_tensor(ri), torch.as_tensor(rh)].contiguous()
    out, _ = oracle.ssa_rows(qr, k, v, rb, rh, ri, Hq=Hq, n_sink=ns, window=win, scale=scale, block=block)
    return float((out * dout.double().numpy().reshape(out.shape)).sum())


def test_gradients_match_central_differences_of_the_forward():
    B, S, Hq, Hkv, d, dv, ns, win, block, scale = 1, 14, 2, 1, 4, 3, 1, 2, 3, 0.6
    q, k, v, dout = _rand((B, S, Hq, d), 21), _rand((B, S, Hkv, d), 22), _rand((B, S, Hkv, dv), 23), _rand((B, S, Hq, dv), 24)
    dq, dk, dvv = oracle.ssa_backward(q, k, v, dout, n_sink=ns, window=win, scale=scale, block=block)
    eps = 2.0 ** -7     # exactly representable steps: the fp32 inputs move by exactly eps
    rng = np.random.default_rng(0)
    for name, t, g in (("q", q, dq), ("k", k, dk), ("v", v, dvv)):
        for _ in range(12):
            idx = tuple(int(rng.integers(0, n)) for n in t.shape)
            tp, tm = t.clone(), t.clone()
            tp[idx] += eps
            tm[idx] -= eps
            args = {"q": q, "k": k, "v": v}
            fp = _forward_loss(**{**args, name: tp}, dout=dout, ns=ns, win=win, block=block, scale=scale)
            fm = _forward_loss(**{**args, name: tm}, dout=dout, ns=ns, win=win, block=block, scale=scale)
            fd = (fp - fm) / (2 * eps)
            assert abs(fd - g[idx]) < 5e-4 * max(1.0, abs(g[idx])), (name, idx, fd, g[idx])


def test_zero_queries_closed_form():
    """Q = 0: uniform weights 1/|live(i)|, so dV_j = sum_i dO_i / |live(i)|, dK = 0, and
    dQ_i = scale * sum_j (dO_i.v_j - mean) k_j / |live(i)|."""
    B, S, Hq, d, dv, ns, win, scale = 1, 30, 1, 5, 4, 2, 6, 0.7
    q = torch.zeros(B, S, Hq, d)
    k, v, dout = _rand((B, S, 1, d), 31), _rand((B, S, 1, dv), 32), _rand((B, S, Hq, dv), 33)
    dq, dk, dvv = oracle.ssa_backward(q, k, v, dout, n_sink=ns, window=win, scale=scale)
    kd, vd, dd = k.double().numpy()[0, :, 0], v.double().numpy()[0, :, 0], dout.double().numpy()[0, :, 0]
    want_dv = np.zeros((S, dv))
    want_dq = np.zeros((S, d))
    for i in range(S):
        live = sorted(_set_live(i, ns, win, None))
        n = len(live)
        dP = np.array([dd[i] @ vd[j] for j in live])
        for j, x in zip(live, dP):
            want_dv[j] += dd[i] / n
            want_dq[i] += scale * (x - dP.mean()) / n * kd[j]
    np.testing.assert_allclose(dvv[0, :, 0], want_dv, atol=1e-12)
    np.testing.assert_allclose(dq[0, :, 0], want_dq, atol=1e-12)
    assert np.abs(dk).max() == 0.0


def test_dk_summed_over_the_keys_of_a_single_query_head_group_vanishes():
    """Adding one vector c to every key shifts all scores of a row by q.c and changes nothing in the
    softmax; hence sum_j dS_ij = 0 for every row, and the sum of dK over all keys, which is
    scale * sum_i (sum_j dS_ij) q_i, is zero."""
    B, S, Hq, d, dv, ns, win, scale = 1, 25, 2, 6, 5, 1, 4, 0.5
    q, k, v, dout = _rand((B, S, Hq, d), 41), _rand((B, S, 1, d), 42), _rand((B, S, 1, dv), 43), _rand((B, S, Hq, dv), 44)
    dq, dk, _ = oracle.ssa_backward(q, k, v, dout, n_sink=ns, window=win, scale=scale)
    assert np.abs(dk.sum(axis=1)).max() < 1e-12


def test_rows_without_dout_contribute_nothing_and_get_zero_dq():
    B, S, Hq, d, dv, ns, win, scale = 1, 40, 2, 6, 5, 2, 5, 0.5
    q, k, v, dout = _rand((B, S, Hq, d), 51), _rand((B, S, 1, d), 52), _rand((B, S, 1, dv), 53), _rand((B, S, Hq, dv), 54)
    keep = torch.zeros(B, S, Hq, 1)
    keep[0, 7, 1] = 1
    keep[0, 33, 0] = 1
    sparse = dout * keep
    dq, dk, dvv = oracle.ssa_backward(q, k, v, sparse, n_sink=ns, window=win, scale=scale)
    rq, rk, rv = _autograd(q, k, v, sparse, ns, win, None, scale)
    np.testing.assert_allclose(dq, rq, atol=1e-12)
    np.testing.assert_allclose(dk, rk, atol=1e-12)
    np.testing.assert_allclose(dvv, rv, atol=1e-12)
    assert np.abs(dq[0, :7]).max() == 0.0 and np.count_nonzero(np.abs(dq).sum(-1)) == 2


def test_saved_forward_of_its_own_gives_the_gradient_and_the_substitution_is_the_stated_one():
    """With the forward's own out and lse handed in, nothing changes (up to their fp32 storage); with
    other values, D_i = dO_i . out_i and p_ij = exp(scale q_i.k_j - lse_i) are what enter: checked on
    dV, which is sum_i p_ij dO_i and so scales by exp(-shift) when every lse is shifted, and on dQ
    through the closed form for one query row."""
    B, S, Hq, d, dv, ns, win, scale = 1, 30, 2, 6, 5, 2, 7, 0.5
    q, k, v, dout = _rand((B, S, Hq, d), 61), _rand((B, S, 1, d), 62), _rand((B, S, 1, dv), 63), _rand((B, S, Hq, dv), 64)
    b, i, h = np.meshgrid(np.arange(B), np.arange(S), np.arange(Hq), indexing="ij")
    rb, ri, rh = b.ravel(), i.ravel(), h.ravel()
    qr = q[torch.as_tensor(rb), torch.as_tensor(ri), torch.as_tensor(rh)].contiguous()
    o, l = oracle.ssa_rows(qr, k, v, rb, rh, ri, Hq=Hq, n_sink=ns, window=win, scale=scale)
    out = torch.as_tensor(o.reshape(B, S, Hq, dv)).float()
    lse = torch.as_tensor(l.reshape(B, S, Hq)).permute(0, 2, 1).contiguous().float()
    base = oracle.ssa_backward(q, k, v, dout, n_sink=ns, window=win, scale=scale)
    same = oracle.ssa_backward(q, k, v, dout, n_sink=ns, window=win, scale=scale, out=out, lse=lse)
    for x, y in zip(base, same):
        np.testing.assert_allclose(x, y, atol=2e-6)      # out and lse went through fp32
    shifted = oracle.ssa_backward(q, k, v, dout, n_sink=ns, window=win, scale=scale, out=out, lse=lse + 1.0)
    np.testing.assert_allclose(shifted[2], same[2] * np.exp(-1.0), atol=2e-6)   # lse + 1 is rounded to fp32
    # one row, out replaced by zeros: D = 0, so dQ_i = scale sum_j p_ij (dO_i . v_j) k_j
    keep = torch.zeros(B, S, Hq, 1)
    keep[0, 11, 1] = 1
    zero_out = oracle.ssa_backward(q, k, v, dout * keep, n_sink=ns, window=win, scale=scale, out=out * 0, lse=lse)
    live = sorted(_set_live(11, ns, win, None))
    s = np.array([scale * float(q[0, 11, 1].double() @ k[0, j, 0].double()) for j in live])
    pj = np.exp(s - float(lse[0, 1, 11]))
    want = sum(scale * pj[n] * float(dout[0, 11, 1].double() @ v[0, j, 0].double()) * k[0, j, 0].double().numpy()
               for n, j in enumerate(live))
    np.testing.assert_allclose(zero_out[0][0, 11, 1], want, atol=1e-9)


def test_listed_rows_form_equals_the_dense_form_with_zeros_elsewhere():
    B, S, Hq, d, dv, ns, win, block, scale = 2, 40, 4, 6, 5, 1, 2, 4, 0.5
    q, k, v, dout = _rand((B, S, Hq, d), 71), _rand((B, S, 2, d), 72), _rand((B, S, 2, dv), 73), _rand((B, S, Hq, dv), 74)
    rb = np.array([0, 1, 1, 0, 0]); rh = np.array([3, 0, 2, 1, 3]); ri = np.array([5, 39, 0, 17, 17])
    keep = torch.zeros(B, S, Hq, 1)
    keep[torch.as_tensor(rb), torch.as_tensor(ri), torch.as_tensor(rh)] = 1
    dense = oracle.ssa_backward(q, k, v, dout * keep, n_sink=ns, window=win, scale=scale, block=block)
    idx = (torch.as_tensor(rb), torch.as_tensor(ri), torch.as_tensor(rh))
    dq_rows, dk, dvv = oracle.ssa_backward_rows(q[idx].contiguous(), k, v, dout[idx].contiguous(), rb, rh, ri, Hq=Hq,
                                                 n_sink=ns, window=win, scale=scale, block=block)
    np.testing.assert_allclose(dq_rows, dense[0][rb, ri, rh], atol=1e-14)
    np.testing.assert_allclose(dk, dense[1], atol=1e-14)
    np.testing.assert_allclose(dvv, dense[2], atol=1e-14)


def test_backward_arguments_are_checked():
    q, k, v, dout = _rand((1, 4, 1, 4), 1), _rand((1, 4, 1, 4), 2), _rand((1, 4, 1, 4), 3), _rand((1, 4, 1, 4), 4)
    with pytest.raises(RuntimeError):
        oracle.ssa_backward(q, k, v, dout, n_sink=-1, window=2, scale=1.0)
    with pytest.raises(RuntimeError):
        oracle.ssa_backward(q, k, v, dout, n_sink=0, window=0, scale=1.0)
