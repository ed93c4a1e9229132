"""Pins of the fp64 oracle against things other than itself (CPU only).

What fixes the expected values here: hand-enumerated live sets (tests/golden), the paper's own
block arithmetic (Training section), torch's scaled_dot_product_attention as an independent
library routine for the window >= S reduction (Eq. 2 -> Eq. 1) and for brute-force boolean masks
built from Python sets, and closed forms (single-key rows, Q = 0, constant V, score shift).
"""
from pathlib import Path

import numpy as np
import pytest
import torch

import oracle

GOLD = Path(__file__).resolve().parent / "golden"


def _rows_all(B, H, S):
    b, h, i = np.meshgrid(np.arange(B), np.arange(H), np.arange(S), indexing="ij")
    return b.ravel(), h.ravel(), i.ravel()


def _gather_q(q, rb, rh, ri):
    # q [B, S, Hq, d] -> [n, d]
    return q[torch.as_tensor(rb), torch.as_tensor(ri), torch.as_tensor(rh)].contiguous()


def _oracle_full(q, k, v, n_sink, window, scale, **kw):
    """Oracle on every (b, h, i); returns out [B, S, Hq, d_v], lse [B, Hq, S]."""
    B, S, Hq, _ = q.shape
    rb, rh, ri = _rows_all(B, Hq, S)
    res = oracle.ssa_rows(_gather_q(q, rb, rh, ri), k, v, rb, rh, ri, Hq=Hq, n_sink=n_sink,
                          window=window, scale=scale, **kw)
    d_v = res[0].shape[1]
    out = res[0].reshape(B, Hq, S, d_v).transpose(0, 2, 1, 3)
    lse = res[1].reshape(B, Hq, S)
    return (out, lse) + tuple(res[2:])


def _set_live(i, n_sink, window):
    """The live set from its verbal definition, with Python sets (independent of the oracle)."""
    return set(range(0, min(n_sink, i + 1))) | set(range(max(0, i - window + 1), i + 1))


def _sdpa_masked(q, k, v, n_sink, window, scale):
    """Library attention under a boolean mask built key by key from Python sets (fp64)."""
    B, S, Hq, _ = q.shape
    Hkv = k.shape[2]
    mask = torch.zeros(S, S, dtype=torch.bool)
    for i in range(S):
        for j in _set_live(i, n_sink, window):
            mask[i, j] = True
    qd = q.double().permute(0, 2, 1, 3)
    kd = k.double().permute(0, 2, 1, 3).repeat_interleave(Hq // Hkv, dim=1)
    vd = v.double().permute(0, 2, 1, 3).repeat_interleave(Hq // Hkv, dim=1)
    o = torch.nn.functional.scaled_dot_product_attention(qd, kd, vd, attn_mask=mask, scale=scale)
    return o.permute(0, 2, 1, 3).numpy()


def _rand(shape, seed, dtype=torch.float32):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(shape, generator=g, dtype=torch.float32).to(dtype)


# ---------------------------------------------------------------- index set ----------------

def _hand_cases():
    for line in (GOLD / "hand_live_sets.txt").read_text().splitlines():
        if not line.strip() or line.startswith("#"):
            continue
        left, right = line.split(":")
        S, ns, W, i = (int(x) for x in left.split())
        yield S, ns, W, i, sorted(int(x) for x in right.split())


@pytest.mark.parametrize("S,ns,W,i,live", list(_hand_cases()))
def test_live_mask_hand_enumerated(S, ns, W, i, live):
    m = oracle.live_mask(i, S, ns, W)
    assert sorted(np.nonzero(m)[0].tolist()) == live


@pytest.mark.parametrize("S,ns,W,i,live", list(_hand_cases()))
def test_weights_support_is_hand_enumerated_set(S, ns, W, i, live):
    q = _rand((1, S, 1, 4), 1)
    k = _rand((1, S, 1, 4), 2)
    v = _rand((1, S, 1, 3), 3)
    _, _, w = oracle.ssa_rows(q[0, i:i + 1, 0], k, v, [0], [0], [i], Hq=1, n_sink=ns, window=W,
                              scale=0.5, want_weights=True)
    assert sorted(np.nonzero(w[0])[0].tolist()) == live
    assert abs(w[0].sum() - 1.0) < 1e-12


def test_paper_block_arithmetic():
    b, s, l, total = (int(x) for x in (GOLD / "ssa_block_params.txt").read_text().splitlines()[-1].split())
    ns, W = s * b, l * b
    assert ns + W == total
    S = 4096
    for i in (S - 1, 3000, total, total - 1):
        assert int(oracle.live_mask(i, S, ns, W).sum()) == total
    assert int(oracle.live_mask(total - 2, S, ns, W).sum()) == total - 1


@pytest.mark.parametrize("S,ns,W", [(50, 0, 1), (50, 3, 7), (64, 8, 16), (40, 64, 5), (33, 4, 1000), (97, 5, 92)])
def test_live_count_and_pair_closed_form(S, ns, W):
    T = ns + W
    for i in range(S):
        m = oracle.live_mask(i, S, ns, W)
        assert int(m.sum()) == min(i + 1, T)
        assert set(np.nonzero(m)[0].tolist()) == _set_live(i, ns, W)
    closed = T * (T + 1) // 2 + (S - T) * T if S >= T else S * (S + 1) // 2
    assert oracle.count_pairs(S, ns, W) == closed


@pytest.mark.parametrize("S,ns,W", [(50, 0, 1), (50, 3, 7), (64, 8, 16), (40, 64, 5), (33, 4, 1000), (300, 128, 100)])
def test_closed_form_live_count_of_the_gpu_probes(S, ns, W):
    """The closed form the full-size index-set probes compare every row's log-sum-exp with."""
    from tests import helpers as H
    i = np.arange(S, dtype=np.int64)
    want = np.asarray([int(oracle.live_mask(int(x), S, ns, W).sum()) for x in i])
    assert (H.live_count_tokens(i, ns, W) == want).all()


def test_pair_counts_of_the_workloads():
    # closed form at the real sizes; the one-by-one count is checked at the smallest of them
    assert oracle.count_pairs(1024, 64, 256) == 276_640
    T = 4224
    assert T * (T + 1) // 2 + (32768 - T) * T == 129_493_056
    T = 8320
    assert T * (T + 1) // 2 + (131072 - T) * T == 1_055_912_000
    assert T * (T + 1) // 2 + (1048576 - T) * T == 8_689_545_280


# ---------------------------------------------------------------- values -------------------

@pytest.mark.parametrize("Hq,Hkv", [(1, 1), (4, 4), (4, 2), (6, 1)])
def test_window_at_least_S_is_textbook_causal_attention(Hq, Hkv):
    B, S, d, dv = 2, 37, 16, 12
    q, k, v = _rand((B, S, Hq, d), 10), _rand((B, S, Hkv, d), 11), _rand((B, S, Hkv, dv), 12)
    scale = 0.3
    for ns, W in [(0, S), (5, S + 3), (0, oracle.INT64_MAX), (S + 9, 1)]:
        out, lse = _oracle_full(q, k, v, ns, W, scale)
        qd = q.double().permute(0, 2, 1, 3)
        kd = k.double().permute(0, 2, 1, 3).repeat_interleave(Hq // Hkv, dim=1)
        vd = v.double().permute(0, 2, 1, 3).repeat_interleave(Hq // Hkv, dim=1)
        ref = torch.nn.functional.scaled_dot_product_attention(qd, kd, vd, is_causal=True, scale=scale)
        np.testing.assert_allclose(out, ref.permute(0, 2, 1, 3).numpy(), rtol=0, atol=1e-12)
        s = torch.einsum("bhid,bhjd->bhij", qd, kd) * scale
        s = s.masked_fill(torch.triu(torch.ones(S, S, dtype=torch.bool), 1), float("-inf"))
        np.testing.assert_allclose(lse, torch.logsumexp(s, -1).numpy(), rtol=0, atol=1e-12)


@pytest.mark.parametrize("ns,W", [(0, 1), (0, 5), (3, 4), (8, 8), (2, 31), (40, 3)])
@pytest.mark.parametrize("Hq,Hkv", [(1, 1), (4, 2)])
def test_matches_library_attention_under_set_built_mask(ns, W, Hq, Hkv):
    B, S, d, dv = 1, 33, 8, 5
    q, k, v = _rand((B, S, Hq, d), 20), _rand((B, S, Hkv, d), 21), _rand((B, S, Hkv, dv), 22)
    out, _ = _oracle_full(q, k, v, ns, W, 0.7)
    np.testing.assert_allclose(out, _sdpa_masked(q, k, v, ns, W, 0.7), rtol=0, atol=1e-12)


def test_row_zero_and_single_key_rows():
    S, d, dv = 9, 6, 4
    q, k, v = _rand((1, S, 1, d), 30), _rand((1, S, 1, d), 31), _rand((1, S, 1, dv), 32)
    out, lse = _oracle_full(q, k, v, 0, 1, 1.25)  # window 1, no sink: every row sees only itself
    np.testing.assert_allclose(out[0, :, 0], v[0, :, 0].double().numpy(), atol=1e-15)
    dots = (q[0, :, 0].double() * k[0, :, 0].double()).sum(-1).numpy() * 1.25
    np.testing.assert_allclose(lse[0, 0], dots, atol=1e-13)
    out, lse = _oracle_full(q, k, v, 3, 4, 1.25)  # any pattern: row 0 sees key 0 only
    np.testing.assert_allclose(out[0, 0, 0], v[0, 0, 0].double().numpy(), atol=1e-15)
    assert abs(lse[0, 0, 0] - dots[0]) < 1e-13


def test_zero_queries_give_uniform_weights():
    S, ns, W = 41, 3, 6
    k, v = _rand((1, S, 1, 8), 41), _rand((1, S, 1, 5), 42)
    q = torch.zeros(1, S, 1, 8)
    out, lse = _oracle_full(q, k, v, ns, W, 0.9)
    for i in range(S):
        live = sorted(_set_live(i, ns, W))
        np.testing.assert_allclose(out[0, i, 0], v[0, live, 0].double().mean(0).numpy(), atol=1e-13)
        assert abs(lse[0, 0, i] - np.log(min(i + 1, ns + W))) < 1e-13


def test_constant_values_and_score_shift():
    S, ns, W, d = 29, 2, 5, 7
    q, k = _rand((1, S, 1, d), 50), _rand((1, S, 1, d), 51)
    v = torch.full((1, S, 1, 3), 0.625)
    out, lse = _oracle_full(q, k, v, ns, W, 0.4)
    np.testing.assert_allclose(out, 0.625, atol=1e-14)
    # one more feature that is 1 in every key and c/scale in every query adds c to every score
    c = 1.75
    v2 = _rand((1, S, 1, 3), 52)
    out_a, lse_a = _oracle_full(q, k, v2, ns, W, 0.4)
    q2 = torch.cat([q, torch.full((1, S, 1, 1), c / 0.4)], -1)
    k2 = torch.cat([k, torch.ones(1, S, 1, 1)], -1)
    out_b, lse_b = _oracle_full(q2, k2, v2, ns, W, 0.4)
    np.testing.assert_allclose(out_b, out_a, atol=1e-12)
    np.testing.assert_allclose(lse_b, lse_a + c, atol=1e-6)  # c/0.4 is rounded to fp32


def test_weights_rows_sum_to_one_and_vanish_outside_live_set():
    S, ns, W = 64, 4, 9
    q, k, v = _rand((1, S, 2, 8), 60), _rand((1, S, 1, 8), 61), _rand((1, S, 1, 4), 62)
    _, _, w = _oracle_full(q, k, v, ns, W, 0.5, want_weights=True)
    w = w.reshape(1, 2, S, S)
    for i in range(S):
        live = _set_live(i, ns, W)
        for h in range(2):
            assert abs(w[0, h, i].sum() - 1.0) < 1e-12
            assert set(np.nonzero(w[0, h, i])[0].tolist()) == live


def test_operands_are_not_interchangeable():
    # a transposed / swapped operand, a dropped scale or a wrong head map must change the result
    B, S, Hq, Hkv, d = 1, 12, 4, 2, 6
    q, k, v = _rand((B, S, Hq, d), 70), _rand((B, S, Hkv, d), 71), _rand((B, S, Hkv, d), 72)
    base = _sdpa_masked(q, k, v, 2, 3, 0.8)
    ours, _ = _oracle_full(q, k, v, 2, 3, 0.8)
    np.testing.assert_allclose(ours, base, atol=1e-12)
    for wrong in (_sdpa_masked(q, v, k, 2, 3, 0.8), _sdpa_masked(q, k, v, 2, 3, 1.0),
                  _sdpa_masked(q, k, v, 3, 3, 0.8), _sdpa_masked(q, k, v, 2, 4, 0.8),
                  _sdpa_masked(q, k.flip(2), v.flip(2), 2, 3, 0.8)):
        assert np.abs(ours - wrong).max() > 1e-3


def test_bf16_inputs_are_widened_exactly_and_mla_alias():
    S, Hq, d, dv = 21, 3, 16, 8
    q, kv = _rand((1, S, Hq, d), 80, torch.bfloat16), _rand((1, S, 1, d), 81, torch.bfloat16)
    rb, rh, ri = _rows_all(1, Hq, S)
    out, lse = oracle.ssa_rows(_gather_q(q, rb, rh, ri), kv, ("alias", dv), rb, rh, ri, Hq=Hq,
                               n_sink=2, window=5, scale=0.25)
    out = out.reshape(1, Hq, S, dv).transpose(0, 2, 1, 3)
    ref = _sdpa_masked(q.float(), kv.float(), kv.float()[..., :dv].contiguous(), 2, 5, 0.25)
    np.testing.assert_allclose(out, ref, atol=1e-12)


def test_decode_row_is_last_prefill_row_of_a_longer_cache():
    # a cache with S_max rows of which L are valid: rows j >= L are never alive for i = L - 1
    S_max, L, d, dv, Hq = 40, 23, 8, 8, 2
    q_all, cache = _rand((1, S_max, Hq, d), 90), _rand((1, S_max, 1, d), 91)
    vcache = _rand((1, S_max, 1, dv), 92)
    i = L - 1
    out_c, lse_c = oracle.ssa_rows(q_all[0, i], cache, vcache, [0, 0], [0, 1], [i, i], Hq=Hq,
                                   n_sink=3, window=6, scale=0.35)
    out_p, lse_p = oracle.ssa_rows(q_all[0, i], cache[:, :L].contiguous(), vcache[:, :L].contiguous(),
                                   [0, 0], [0, 1], [i, i], Hq=Hq, n_sink=3, window=6, scale=0.35)
    np.testing.assert_array_equal(out_c, out_p)
    np.testing.assert_array_equal(lse_c, lse_p)
    ref = _sdpa_masked(q_all[:, :L], cache[:, :L], vcache[:, :L], 3, 6, 0.35)
    np.testing.assert_allclose(out_c, ref[0, i], atol=1e-12)


def test_disjoint_key_sets_combine_by_the_log_sum_exp_rule():
    # attention over A u B (disjoint) from attention over A and over B: lse = ln(e^lA + e^lB),
    # out = e^(lA - lse) outA + e^(lB - lse) outB. This identity is what a key-split decode merges
    # with; here it is checked on the oracle itself, the parts being two caches cut from one.
    L, m, d, dv, Hq = 37, 14, 8, 6, 2
    q, cache, vcache = _rand((Hq, d), 70), _rand((1, L, 1, d), 71), _rand((1, L, 1, dv), 72)
    kw = dict(Hq=Hq, n_sink=0, window=oracle.INT64_MAX, scale=0.4)
    full, lse = oracle.ssa_rows(q, cache, vcache, [0, 0], [0, 1], [L - 1, L - 1], **kw)
    oa, la = oracle.ssa_rows(q, cache[:, :m].contiguous(), vcache[:, :m].contiguous(), [0, 0], [0, 1], [m - 1] * 2, **kw)
    ob, lb = oracle.ssa_rows(q, cache[:, m:].contiguous(), vcache[:, m:].contiguous(), [0, 0], [0, 1], [L - m - 1] * 2, **kw)
    merged_lse = np.logaddexp(la, lb)
    merged = np.exp(la - merged_lse)[:, None] * oa + np.exp(lb - merged_lse)[:, None] * ob
    np.testing.assert_allclose(merged_lse, lse, atol=1e-12)
    np.testing.assert_allclose(merged, full, atol=1e-12)


def test_bad_arguments_are_rejected():
    q, k, v = _rand((1, 4, 1, 4), 1), _rand((1, 4, 1, 4), 2), _rand((1, 4, 1, 4), 3)
    with pytest.raises(RuntimeError):
        oracle.ssa_rows(q[0, :1, 0], k, v, [0], [0], [0], Hq=1, n_sink=0, window=0, scale=1.0)
    with pytest.raises(RuntimeError):
        oracle.ssa_rows(q[0, :1, 0], k, v, [0], [0], [4], Hq=1, n_sink=0, window=1, scale=1.0)
