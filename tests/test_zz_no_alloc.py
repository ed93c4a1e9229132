"""loza_ssa_decode_static (the decode entry point that allocates nothing: its partial results live in
a static device buffer of the library) against loza_ssa_decode, through the C ABI: the same bits,
on two calls in a row, the second with a smaller input (the buffer keeps the first call's contents)."""
import numpy as np
import pytest
import torch

import paper_2512_23966_amd as loza
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _rand(shape, seed, device):
    g = torch.Generator(device=device).manual_seed(seed)
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)


def _both(q, kc, lens, ns, win, scale, dev):
    B, Hq, _ = q.shape
    seqlens = torch.tensor(lens, dtype=torch.int32, device=dev)
    out_w, lse_w = H.run_decode(q, kc, kc, seqlens, ns, win, scale, d_v=512)
    out_s = torch.full((B, Hq, 512), float("nan"), dtype=torch.bfloat16, device=dev)
    lse_s = torch.full((B, Hq), float("nan"), dtype=torch.float32, device=dev)
    loza.loza_ssa_decode_static(q, kc, kc, seqlens, out_s, lse_s, ns, win, scale)
    torch.cuda.synchronize()
    return seqlens, (out_w, lse_w), (out_s, lse_s)


def test_static_scratch_decode_equals_workspace_decode_twice(gpu_device):
    dev = gpu_device
    scale = 192 ** -0.5
    # first call: 6 sequences, long caches, many splits
    q1, kc1 = _rand((6, 64, 576), 1, dev), _rand((6, 5000, 1, 576), 2, dev)
    lens1 = [5000, 4999, 2500, 130, 1, 3000]
    sl1, ref1, got1 = _both(q1, kc1, lens1, 128, 2048, scale, dev)
    assert torch.equal(got1[0].view(torch.int16), ref1[0].view(torch.int16))
    assert torch.equal(got1[1].view(torch.int32), ref1[1].view(torch.int32))
    rb, rh = np.repeat(np.arange(6), 64), np.tile(np.arange(64), 6)
    H.compare_decode(q1, kc1, kc1, sl1, got1[0], got1[1], rb, rh, 128, 2048, scale, "static scratch, first call")
    # second call: smaller in every way (fewer sequences, fewer heads, shorter caches, fewer splits)
    q2, kc2 = _rand((2, 16, 576), 3, dev), _rand((2, 700, 1, 576), 4, dev)
    lens2 = [700, 333]
    sl2, ref2, got2 = _both(q2, kc2, lens2, 16, 300, scale, dev)
    assert torch.equal(got2[0].view(torch.int16), ref2[0].view(torch.int16))
    assert torch.equal(got2[1].view(torch.int32), ref2[1].view(torch.int32))
    rb, rh = np.repeat(np.arange(2), 16), np.tile(np.arange(16), 2)
    H.compare_decode(q2, kc2, kc2, sl2, got2[0], got2[1], rb, rh, 16, 300, scale, "static scratch, second call")


def test_static_scratch_rejects_sizes_beyond_its_buffer(gpu_device):
    dev = gpu_device
    B, Hq, S_max = 110, 64, 512   # 110 sequences * 64 heads * 3 splits * 516 floats > 40 MiB
    need = loza.loza_ssa_decode_workspace_bytes(B, Hq, 1, S_max, 512, 128, 2048)
    assert need > loza.LOZA_DECODE_STATIC_BYTES
    q, kc = torch.zeros(B, Hq, 576, dtype=torch.bfloat16, device=dev), torch.zeros(B, S_max, 1, 576, dtype=torch.bfloat16, device=dev)
    out = torch.zeros(B, Hq, 512, dtype=torch.bfloat16, device=dev)
    lse = torch.zeros(B, Hq, dtype=torch.float32, device=dev)
    seqlens = torch.full((B,), S_max, dtype=torch.int32, device=dev)
    with pytest.raises(loza.LozaError) as e:
        loza.loza_ssa_decode_static(q, kc, kc, seqlens, out, lse, 128, 2048, 192 ** -0.5)
    assert e.value.status == -4
