"""Pins of the oracle's block-granular pattern (sink blocks s, local blocks l, block size b:
Architecture section after Eq. 4; s = 1, l = 7, b = 128 in the Training section), CPU only.

The pattern is pinned by the sizes the paper prints, by hand-enumerated live sets, by its b = 1
case (which is the token-granular pattern, pinned elsewhere), by a live set written with Python
sets from the verbal definition, and the values by a library attention routine under that mask.
"""
from pathlib import Path

import numpy as np
import pytest
import torch

import oracle

GOLD = Path(__file__).resolve().parent / "golden"


def _rand(shape, seed, dtype=torch.float32):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(shape, generator=g, dtype=torch.float32).to(dtype)


def _set_live_blocks(i, s, l, b):
    """Live set from the verbal definition: whole sink blocks, the l most recent blocks ending with
    the query's own, nothing after the query."""
    qb = i // b
    keys = set()
    for kb in range(0, s):
        keys |= set(range(kb * b, (kb + 1) * b))
    for kb in range(max(0, qb - l + 1), qb + 1):
        keys |= set(range(kb * b, (kb + 1) * b))
    return {j for j in keys if j <= i}


def _hand_cases():
    for line in (GOLD / "hand_live_sets_blocks.txt").read_text().splitlines():
        if not line.strip() or line.startswith("#"):
            continue
        left, right = line.split(":")
        S, s, l, b, i = (int(x) for x in left.split())
        yield S, s, l, b, i, sorted(int(x) for x in right.split())


@pytest.mark.parametrize("S,s,l,b,i,live", list(_hand_cases()))
def test_block_live_mask_hand_enumerated(S, s, l, b, i, live):
    assert sorted(np.nonzero(oracle.live_mask_blocks(i, S, s, l, b))[0].tolist()) == live


@pytest.mark.parametrize("S,s,l,b,i,live", list(_hand_cases()))
def test_block_weights_support_is_hand_enumerated_set(S, s, l, b, i, live):
    q, k, v = _rand((1, S, 1, 4), 1), _rand((1, S, 1, 4), 2), _rand((1, S, 1, 3), 3)
    _, _, w = oracle.ssa_rows(q[0, i:i + 1, 0], k, v, [0], [0], [i], Hq=1, n_sink=s, window=l, block=b,
                              scale=0.5, want_weights=True)
    assert sorted(np.nonzero(w[0])[0].tolist()) == live
    assert abs(w[0].sum() - 1.0) < 1e-12


def test_paper_sizes_give_at_most_1024_live_tokens():
    b, s, l, total = (int(x) for x in (GOLD / "ssa_block_params.txt").read_text().splitlines()[-1].split())
    S = 4096
    counts = [int(oracle.live_mask_blocks(i, S, s, l, b).sum()) for i in range(S)]
    assert max(counts) == total == 1024
    # the count is i + 1 while everything is visible, then runs through (s + l - 1) b + 1 ... (s + l) b
    # once per block: full at the last query of a block, lowest at the first
    assert counts[:total] == list(range(1, total + 1))
    for i in range(total, S):
        assert counts[i] == (s + l - 1) * b + (i % b) + 1
    assert counts[2047] == 1024 and counts[2048] == 897


@pytest.mark.parametrize("S,s,l,b", [(40, 1, 2, 4), (37, 0, 1, 5), (64, 2, 3, 8), (50, 1, 7, 128), (29, 3, 1, 2), (30, 1, 4, 1),
                                     (1300, 1, 7, 128), (200, 3, 2, 16), (90, 5, 1, 8)])
def test_closed_form_block_live_count_of_the_gpu_probes(S, s, l, b):
    """The closed form the full-size index-set probe compares every row's log-sum-exp with."""
    from tests import helpers as H
    i = np.arange(S, dtype=np.int64)
    want = np.asarray([int(oracle.live_mask_blocks(int(x), S, s, l, b).sum()) for x in i])
    assert (H.live_count_blocks(i, s, l, b) == want).all()


@pytest.mark.parametrize("S,s,l,b", [(40, 1, 2, 4), (37, 0, 1, 5), (64, 2, 3, 8), (50, 1, 7, 128), (29, 3, 1, 2), (30, 1, 4, 1)])
def test_block_mask_equals_set_definition_and_pair_count(S, s, l, b):
    n = 0
    for i in range(S):
        live = _set_live_blocks(i, s, l, b)
        assert set(np.nonzero(oracle.live_mask_blocks(i, S, s, l, b))[0].tolist()) == live
        n += len(live)
    assert oracle.count_pairs_blocks(S, s, l, b) == n


@pytest.mark.parametrize("ns,W", [(0, 1), (3, 5), (2, 100), (7, 3)])
def test_block_size_one_is_the_token_granular_pattern(ns, W):
    S, Hq = 23, 2
    q, k, v = _rand((1, S, Hq, 6), 11), _rand((1, S, 1, 6), 12), _rand((1, S, 1, 5), 13)
    rb = np.zeros(S * Hq, dtype=np.int64)
    rh = np.repeat(np.arange(Hq), S)
    ri = np.tile(np.arange(S), Hq)
    qr = q[0, torch.as_tensor(ri), torch.as_tensor(rh)].contiguous()
    a = oracle.ssa_rows(qr, k, v, rb, rh, ri, Hq=Hq, n_sink=ns, window=W, scale=0.3, want_weights=True)
    c = oracle.ssa_rows(qr, k, v, rb, rh, ri, Hq=Hq, n_sink=ns, window=W, block=1, scale=0.3, want_weights=True)
    for x, y in zip(a, c):
        np.testing.assert_array_equal(x, y)


@pytest.mark.parametrize("s,l,b,Hq,Hkv", [(1, 2, 4, 1, 1), (1, 3, 8, 4, 2), (0, 2, 5, 2, 2), (2, 1, 3, 2, 1)])
def test_block_values_match_library_attention_under_set_built_mask(s, l, b, Hq, Hkv):
    S, d, dv, scale = 45, 8, 6, 0.37
    q, k, v = _rand((1, S, Hq, d), 21), _rand((1, S, Hkv, d), 22), _rand((1, S, Hkv, dv), 23)
    mask = torch.zeros(S, S, dtype=torch.bool)
    for i in range(S):
        for j in _set_live_blocks(i, s, l, b):
            mask[i, j] = True
    qd = q.double().permute(0, 2, 1, 3)
    kd = k.double().permute(0, 2, 1, 3).repeat_interleave(Hq // Hkv, dim=1)
    vd = v.double().permute(0, 2, 1, 3).repeat_interleave(Hq // Hkv, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(qd, kd, vd, attn_mask=mask, scale=scale)
    ref = ref.permute(0, 2, 1, 3).numpy()
    b_, h_, i_ = np.meshgrid(np.arange(1), np.arange(Hq), np.arange(S), indexing="ij")
    rb, rh, ri = b_.ravel(), h_.ravel(), i_.ravel()
    qr = q[torch.as_tensor(rb), torch.as_tensor(ri), torch.as_tensor(rh)].contiguous()
    out, lse = oracle.ssa_rows(qr, k, v, rb, rh, ri, Hq=Hq, n_sink=s, window=l, block=b, scale=scale)
    np.testing.assert_allclose(out.reshape(Hq, S, dv).transpose(1, 0, 2), ref[0], atol=1e-12)
    # lse against the mask-restricted log-sum-exp of the scaled scores
    sc = scale * torch.einsum("bhid,bhjd->bhij", qd, kd)
    sc = sc.masked_fill(~mask, float("-inf"))
    np.testing.assert_allclose(lse.reshape(Hq, S), torch.logsumexp(sc, dim=-1)[0].numpy(), atol=1e-12)


def test_block_arguments_are_checked():
    q, k, v = _rand((1, 4, 1, 4), 1), _rand((1, 4, 1, 4), 2), _rand((1, 4, 1, 4), 3)
    for s, l, b in ((0, 0, 2), (-1, 1, 2), (1, 1, 0)):
        with pytest.raises(RuntimeError):
            oracle.ssa_rows(q[0, :1, 0], k, v, [0], [0], [0], Hq=1, n_sink=s, window=l, block=b, scale=1.0)


# ---- calibration blend (Eq. 3) -------------------------------------------------------------------

def _calib_case(alpha, s=1, l=2, b=4, S=40, Hq=2, d=8, dv=5, scale=0.3):
    q, k, v = _rand((1, S, Hq, d), 31), _rand((1, S, 1, d), 32), _rand((1, S, 1, dv), 33)
    rb = np.zeros(S * Hq, dtype=np.int64)
    rh = np.repeat(np.arange(Hq), S)
    ri = np.tile(np.arange(S), Hq)
    qr = q[0, torch.as_tensor(ri), torch.as_tensor(rh)].contiguous()
    res = oracle.calibration_rows(qr, k, v, rb, rh, ri, Hq=Hq, sink_blocks=s, local_blocks=l, block=b, alpha=alpha,
                                  scale=scale)
    return (q, k, v, rh, ri), res


def test_calibration_end_points_are_the_two_attentions():
    _, (blend1, full, sparse, _, _) = _calib_case(1.0)
    _, (blend0, _, _, _, _) = _calib_case(0.0)
    np.testing.assert_array_equal(blend1, full)
    np.testing.assert_array_equal(blend0, sparse)
    assert np.abs(full - sparse).max() > 1e-3  # the two really differ on this input


def test_calibration_is_the_straight_line_between_them():
    _, (mid, full, sparse, _, _) = _calib_case(0.25)
    np.testing.assert_allclose(mid, sparse + 0.25 * (full - sparse), atol=1e-15)


def test_calibration_rows_that_see_their_whole_prefix_do_not_depend_on_alpha():
    (q, k, v, rh, ri), (a, full, sparse, lf, ls) = _calib_case(0.7, s=1, l=2, b=4)
    whole = ri < (1 + 2 - 1) * 4   # every key up to the query is in a sink or local block
    np.testing.assert_allclose(a[whole], full[whole], atol=1e-15)
    np.testing.assert_allclose(lf[whole], ls[whole], atol=1e-15)
    assert np.abs(a[~whole] - full[~whole]).max() > 1e-4


def test_calibration_against_library_attention_under_set_built_masks():
    alpha, s, l, b, scale = 0.4, 1, 2, 4, 0.3
    (q, k, v, rh, ri), (blend, _, _, _, _) = _calib_case(alpha, s, l, b, scale=scale)
    S, Hq = q.shape[1], q.shape[2]
    sparse_mask = torch.zeros(S, S, dtype=torch.bool)
    for i in range(S):
        for j in _set_live_blocks(i, s, l, b):
            sparse_mask[i, j] = True
    qd = q.double().permute(0, 2, 1, 3)
    kd = k.double().permute(0, 2, 1, 3).repeat_interleave(Hq, dim=1)
    vd = v.double().permute(0, 2, 1, 3).repeat_interleave(Hq, dim=1)
    full = torch.nn.functional.scaled_dot_product_attention(qd, kd, vd, is_causal=True, scale=scale)
    sparse = torch.nn.functional.scaled_dot_product_attention(qd, kd, vd, attn_mask=sparse_mask, scale=scale)
    ref = (alpha * full + (1 - alpha) * sparse)[0].numpy()          # [Hq, S, dv]
    np.testing.assert_allclose(blend.reshape(Hq, S, -1), ref, atol=1e-12)


def test_alpha_gradient_is_the_slope_of_the_blend():
    """d/d(alpha) of sum(dout * blend(alpha)) by the difference of two blends (the blend is linear in
    alpha, so the difference quotient is exact up to rounding), and two closed forms."""
    _, (b0, full, sparse, _, _) = _calib_case(0.2)
    _, (b1, _, _, _, _) = _calib_case(0.7)
    dout = np.random.default_rng(5).standard_normal(full.shape)
    slope = (np.sum(dout * b1) - np.sum(dout * b0)) / 0.5
    got = oracle.calibration_alpha_grad(dout, full, sparse)
    assert abs(got - slope) <= 1e-12 * max(1.0, abs(slope))
    assert oracle.calibration_alpha_grad(dout, full, full) == 0.0
    assert oracle.calibration_alpha_grad(np.ones_like(full), full, np.zeros_like(full)) == pytest.approx(full.sum(), rel=1e-14)
    # bf16 and float32 tensors are widened exactly
    t = torch.tensor([[1.5, -2.0], [0.25, 3.0]])
    assert oracle.calibration_alpha_grad(t.to(torch.bfloat16), t, torch.zeros(2, 2)) == 1.5 ** 2 + 4.0 + 0.0625 + 9.0
