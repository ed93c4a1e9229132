"""Rows whose softmax weight sits on one or two keys, far from the start of the sequence.

Such rows are where the rounding of the weights to bf16 shows most (nothing averages it out) and
where the result is as large as single value rows, so that its own rounding to bf16 leaves the
least room (half an ulp is 2^-7 from magnitude 2 on). The kernels compute every result of magnitude
2 and more with unrounded weights (two bf16 terms in the prefill and extend kernel, fp32 in the
decode's merge kernel); these cases make sure that path is taken and holds the bound.
Construction: queries are a multiple of one live key plus noise, the multiple growing over the
heads, so that the weight of that key runs from a few per cent to nearly one.
"""
import numpy as np
import pytest
import torch

from tests import helpers as H
from tests import test_gpu_parity_extend as E

pytestmark = pytest.mark.gpu


def _rand(shape, seed, device):
    g = torch.Generator(device=device).manual_seed(seed)
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)


def _peak(q_rows, key_rows, c_lo, c_hi):
    """q_rows [n, Hq, d] += c_h * key_rows [n, d], c_h rising over the heads."""
    Hq = q_rows.shape[1]
    c = torch.linspace(c_lo, c_hi, Hq, device=q_rows.device)[None, :, None]
    return (q_rows.float() + c * key_rows.float()[:, None, :]).to(torch.bfloat16)


def _n_large(ref_out):
    return int((np.abs(ref_out) >= 2.0).sum())


@pytest.mark.parametrize("S,ns,win,block", [(1400, 128, 700, None), (1145, 2, 1, 128), (900, 0, 300, None)])
def test_mla_prefill_peaked_rows(gpu_device, S, ns, win, block):
    q = _rand((1, S, 64, 576), 11, gpu_device)
    k = _rand((1, S, 1, 576), 12, gpu_device)
    # every 7th query from position 200 on points at a key a little behind it (inside every window here)
    pos = torch.arange(200, S, 7, device=gpu_device)
    q[0, pos] = _peak(q[0, pos], k[0, pos - (pos % 5), 0], 0.02, 0.45)
    scale = 192 ** -0.5
    out, lse = H.run_prefill(q, k, k, ns, win, scale, d_v=512, block=block)
    rb, rh, ri = H.all_rows(1, 64, S)
    ref_out, _ = H.oracle_prefill_rows(q, k, k, rb, rh, ri, ns, win, scale, 512, block)
    assert _n_large(ref_out) > 1000, "the construction no longer produces large results"
    H.compare_prefill(q, k, k, out, lse, rb, rh, ri, ns, win, scale, f"peaked prefill S{S} ns{ns} W{win} b{block}", block=block)


def test_d128_prefill_peaked_rows(gpu_device):
    S, Hq, Hkv, ns, win = 1100, 8, 2, 16, 400
    q = _rand((1, S, Hq, 128), 21, gpu_device)
    k = _rand((1, S, Hkv, 128), 22, gpu_device)
    v = _rand((1, S, Hkv, 128), 23, gpu_device)
    pos = torch.arange(150, S, 3, device=gpu_device)
    for h in range(Hq):
        g = h // (Hq // Hkv)
        q[0, pos, h] = (q[0, pos, h].float() + (0.3 + 0.25 * h) * k[0, pos - 2, g].float()).to(torch.bfloat16)
    scale = 128 ** -0.5
    out, lse = H.run_prefill(q, k, v, ns, win, scale)
    rb, rh, ri = H.all_rows(1, Hq, S)
    ref_out, _ = H.oracle_prefill_rows(q, k, v, rb, rh, ri, ns, win, scale, 128)
    assert _n_large(ref_out) > 1000, "the construction no longer produces large results"
    H.compare_prefill(q, k, v, out, lse, rb, rh, ri, ns, win, scale, "peaked prefill d128")


def test_mla_extend_peaked_rows(gpu_device):
    B, S_max, q_len, lens, ns, win, block = 3, 1145, 114, [1145, 415, 1012], 2, 1, 128
    kc = _rand((B, S_max, 1, 576), 31, gpu_device)
    q = _rand((B, q_len, 64, 576), 32, gpu_device)
    for b, L in enumerate(lens):
        r = torch.arange(0, q_len, 2, device=gpu_device)
        q[b, r] = _peak(q[b, r], kc[b, L - q_len + r, 0], 0.02, 0.45)   # each at its own key (always live)
    seqlens = torch.tensor(lens, dtype=torch.int32, device=gpu_device)
    scale = 192 ** -0.5
    out, lse = E._run(q, kc, kc, seqlens, (ns, win), scale, 512, block)
    E._compare(q, kc, kc, lens, out, lse, (ns, win), scale, "peaked extend", block)
    assert int((out.float().abs() >= 2.0).sum()) > 1000, "the construction no longer produces large results"


@pytest.mark.parametrize("ns,win,block", [(128, 1024, None), (1, 7, 128), (0, None, None)])
def test_mla_decode_peaked_rows(gpu_device, ns, win, block):
    B, S_max, lens = 3, 3000, [3000, 1500, 2047]
    kc = _rand((B, S_max, 1, 576), 41, gpu_device)
    q = _rand((B, 64, 576), 42, gpu_device)
    last = torch.tensor([L - 3 for L in lens], device=gpu_device)
    q = _peak(q, kc[torch.arange(B, device=gpu_device), last, 0], 0.02, 0.6)
    seqlens = torch.tensor(lens, dtype=torch.int32, device=gpu_device)
    scale = 192 ** -0.5
    out, lse = H.run_decode(q, kc, kc, seqlens, ns, win, scale, d_v=512, block=block)
    rb, rh = np.repeat(np.arange(B), 64), np.tile(np.arange(64), B)
    ref_out, _ = H.oracle_decode(q, kc, kc, seqlens, rb, rh, ns, win, scale, 512, block)
    assert _n_large(ref_out) > 100, "the construction no longer produces large results"
    H.compare_decode(q, kc, kc, seqlens, out, lse, rb, rh, ns, win, scale, f"peaked decode ns{ns} W{win} b{block}", block=block)


@pytest.mark.parametrize("S,ns,win", [(640, 128, 300), (600, 0, 2000)])
def test_mla_prefill_scores_that_keep_rising(gpu_device, S, ns, win):
    """Scores that grow with the key position by more than the lazy threshold of the online softmax
    (2^8) per key tile: the reference of every row has to move on almost every tile, so the prefill's
    softmax between the matrix instructions (which takes its exponentials against the current
    reference and checks afterwards) has to take its tiles twice throughout. Keys are noise plus a
    common direction whose weight rises with the position, queries noise plus that direction; the
    direction lives in the 64 features that are not part of the values, so that the results stay
    small and come from the once-rounded weights (no two-term pass beyond the first 128 positions)."""
    g = torch.Generator(device=gpu_device).manual_seed(77)
    d = torch.zeros(576, device=gpu_device)
    d[512:] = torch.randn(64, generator=g, device=gpu_device)
    d = d / d.norm()
    scale = 192 ** -0.5
    # score of key j: about scale * 14 * ramp_j = 0.2 (j - S/2) in natural units: 6.4 per tile of 32 keys = 9.2 in log2 units
    ramp = (torch.arange(S, device=gpu_device, dtype=torch.float32) - S / 2) * (0.2 / (scale * 14.0))
    k = (0.3 * torch.randn(1, S, 1, 576, generator=g, device=gpu_device) + ramp[None, :, None, None] * d).to(torch.bfloat16)
    q = (0.3 * torch.randn(1, S, 64, 576, generator=g, device=gpu_device) + 14.0 * d).to(torch.bfloat16)
    out, lse = H.run_prefill(q, k, k, ns, win, scale, d_v=512)
    rb, rh, ri = H.all_rows(1, 64, S)
    ref_out, ref_lse = H.oracle_prefill_rows(q, k, k, rb, rh, ri, ns, win, scale, 512)
    assert float(np.abs(ref_out).max()) < 1.9, "the construction no longer keeps the results small"
    deep = ri >= 256
    assert float(ref_lse[deep].max() - ref_lse[deep].min()) > 60.0, "the construction no longer makes the scores rise"
    H.compare_prefill(q, k, k, out, lse, rb, rh, ri, ns, win, scale, f"rising scores S{S} ns{ns} W{win}")


def test_mla_prefill_score_jump_that_overflows_the_speculative_weights(gpu_device):
    """Scores that jump by 100 (144 in log2 units) from one key to the next: weights taken against the
    reference of the keys before the jump overflow fp32 (2^128), which the prefill's speculative softmax
    has to notice (an infinite largest weight) and answer by taking the tile again in the ordinary order.
    Same construction as above with a step instead of a ramp: scores of -55 before key 400, +45 from it on."""
    S, ns, win, j_step = 640, 128, 300, 400
    g = torch.Generator(device=gpu_device).manual_seed(78)
    d = torch.zeros(576, device=gpu_device)
    d[512:] = torch.randn(64, generator=g, device=gpu_device)
    d = d / d.norm()
    scale = 192 ** -0.5
    level = torch.where(torch.arange(S, device=gpu_device) < j_step, -55.0, 45.0) / (scale * 14.0)
    k = (0.3 * torch.randn(1, S, 1, 576, generator=g, device=gpu_device) + level[None, :, None, None] * d).to(torch.bfloat16)
    q = (0.3 * torch.randn(1, S, 64, 576, generator=g, device=gpu_device) + 14.0 * d).to(torch.bfloat16)
    out, lse = H.run_prefill(q, k, k, ns, win, scale, d_v=512)
    rb, rh, ri = H.all_rows(1, 64, S)
    ref_out, ref_lse = H.oracle_prefill_rows(q, k, k, rb, rh, ri, ns, win, scale, 512)
    assert float(np.abs(ref_out).max()) < 1.9, "the construction no longer keeps the results small"
    assert float(ref_lse[ri >= j_step].min() - ref_lse[(ri >= 256) & (ri < j_step)].max()) > 80.0, "the construction no longer makes the scores jump past 2^128"
    H.compare_prefill(q, k, k, out, lse, rb, rh, ri, ns, win, scale, "score jump past the fp32 range")


def test_mla_extend_scores_that_keep_rising(gpu_device):
    """The rising scores of the prefill case above through the extend entry point (its own instantiation
    of the tile kernel): 300 new tokens against caches of 640 and 500 rows."""
    B, S_max, q_len, lens, ns, win = 2, 640, 300, [640, 500], 128, 300
    g = torch.Generator(device=gpu_device).manual_seed(79)
    d = torch.zeros(576, device=gpu_device)
    d[512:] = torch.randn(64, generator=g, device=gpu_device)
    d = d / d.norm()
    scale = 192 ** -0.5
    ramp = (torch.arange(S_max, device=gpu_device, dtype=torch.float32) - S_max / 2) * (0.2 / (scale * 14.0))
    kc = (0.3 * torch.randn(B, S_max, 1, 576, generator=g, device=gpu_device) + ramp[None, :, None, None] * d).to(torch.bfloat16)
    q = (0.3 * torch.randn(B, q_len, 64, 576, generator=g, device=gpu_device) + 14.0 * d).to(torch.bfloat16)
    seqlens = torch.tensor(lens, dtype=torch.int32, device=gpu_device)
    out, lse = E._run(q, kc, kc, seqlens, (ns, win), scale, 512, None)
    E._compare(q, kc, kc, lens, out, lse, (ns, win), scale, "rising scores, extend", None)
    assert float(out.float().abs().max()) < 1.9, "the construction no longer keeps the results small"
