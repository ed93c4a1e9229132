"""GPU parity of the fp32 SSA decode against the oracle (1e-5 on out, as for the fp32 prefill)."""
import numpy as np
import pytest
import torch

from tests import helpers as H

pytestmark = pytest.mark.gpu


def _rand(shape, seed, device):
    g = torch.Generator(device=device).manual_seed(seed)
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32)


@pytest.mark.parametrize("B,Hq,Hkv,S_max,d_qk,d_v,alias,lens,ns,win,block", [
    (3, 4, 2, 300, 64, 64, False, [300, 1, 157], 16, 50, None),
    (2, 2, 1, 1100, 96, 64, True, [1100, 640], 64, 256, None),     # values are a prefix of the key rows
    (4, 3, 3, 90, 40, 24, False, [90, 5, 33, 64], 0, 1, None),     # no sink, window of one
    (2, 6, 2, 260, 32, 32, False, [200, 260], 1, 2, 32),           # block-granular
    (2, 1, 1, 128, 256, 256, False, [77, 128], 200, 3, None),      # widest rows, more sink tokens than keys
    (2, 2, 2, 100, 16, 8, False, [100, 50], 3, None, None),        # window = infinity
])
def test_decode_f32(gpu_device, B, Hq, Hkv, S_max, d_qk, d_v, alias, lens, ns, win, block):
    q = _rand((B, Hq, d_qk), 21, gpu_device)
    kc = _rand((B, S_max, Hkv, d_qk), 22, gpu_device)
    vc = kc if alias else _rand((B, S_max, Hkv, d_v), 23, gpu_device)
    # rows at or beyond the length are never read: poison them
    for b, L in enumerate(lens):
        kc[b, L:] = float("nan")
        if not alias:
            vc[b, L:] = float("nan")
    seqlens = torch.tensor(lens, dtype=torch.int32, device=gpu_device)
    scale = d_qk ** -0.5
    out, lse = H.run_decode_f32(q, kc, vc, seqlens, ns, win, scale, d_v=d_v, block=block)
    rb = np.repeat(np.arange(B), Hq)
    rh = np.tile(np.arange(Hq), B)
    H.compare_decode(q, kc, vc, seqlens, out, lse, rb, rh, ns, win, scale, f"f32 decode lens{lens} ns{ns} W{win} b{block}", block=block)


def test_decode_f32_edge_lengths(gpu_device):
    """An empty cache gives out = 0 and lse = -inf; a length beyond the cache is cut to it."""
    B, Hq, S_max, d = 3, 2, 40, 32
    q = _rand((B, Hq, d), 31, gpu_device)
    kc = _rand((B, S_max, 1, d), 32, gpu_device)
    vc = _rand((B, S_max, 1, d), 33, gpu_device)
    seqlens = torch.tensor([0, 1000, 40], dtype=torch.int32, device=gpu_device)
    out, lse = H.run_decode_f32(q, kc, vc, seqlens, 4, 8, d ** -0.5)
    assert torch.all(out[0] == 0) and torch.all(torch.isinf(lse[0]) & (lse[0] < 0))
    out2, lse2 = H.run_decode_f32(q[1:2], kc[1:2], vc[1:2], torch.tensor([40], dtype=torch.int32, device=gpu_device), 4, 8, d ** -0.5)
    assert torch.equal(out[1], out2[0]) and torch.equal(lse[1], lse2[0])


def test_decode_f32_equals_the_last_prefill_row(gpu_device):
    S, Hq, Hkv, d, ns, win = 150, 4, 2, 64, 5, 30
    q = _rand((1, S, Hq, d), 41, gpu_device)
    k = _rand((1, S, Hkv, d), 42, gpu_device)
    v = _rand((1, S, Hkv, d), 43, gpu_device)
    scale = d ** -0.5
    out_p, lse_p = H.run_prefill(q, k, v, ns, win, scale)
    seqlens = torch.tensor([S], dtype=torch.int32, device=gpu_device)
    out_d, lse_d = H.run_decode_f32(q[:, S - 1].contiguous(), k, v, seqlens, ns, win, scale)
    assert torch.equal(out_d[0], out_p[0, S - 1]) and torch.equal(lse_d[0], lse_p[0, :, S - 1])
