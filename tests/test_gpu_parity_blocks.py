"""GPU parity of the block-granular SSA pattern (sink blocks s, local blocks l, block size b:
Architecture section after Eq. 4; b = 128, s = 1, l = 7 in the Training section) against the
oracle's explicit block predicate: element by element at small sizes, the index set bit by bit,
and the paper's own sizes at 128K on sampled rows."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import oracle
from paper_2512_23966_amd import workloads as W
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _rand(shape, seed, dtype, device):
    g = torch.Generator(device=device).manual_seed(seed)
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32).to(dtype)


@pytest.mark.parametrize("B,Hq,Hkv,S,d,s,l,b", [
    (1, 1, 1, 1024, 64, 1, 2, 128),   # the tiny fp32 shape under a block pattern
    (2, 3, 1, 97, 40, 1, 2, 8),       # ragged last block
    (1, 4, 2, 130, 64, 0, 1, 16),     # no sink, own block only
    (1, 2, 2, 70, 32, 2, 3, 1),       # block of one token: the token-granular pattern
    (1, 2, 1, 90, 24, 1, 100, 7),     # more local blocks than the sequence has
    (1, 1, 1, 50, 16, 1, 1, 1000),    # one block holds everything
])
def test_fp32_prefill_blocks(gpu_device, B, Hq, Hkv, S, d, s, l, b):
    q = _rand((B, S, Hq, d), 1, torch.float32, gpu_device)
    k = _rand((B, S, Hkv, d), 2, torch.float32, gpu_device)
    v = _rand((B, S, Hkv, d), 3, torch.float32, gpu_device)
    scale = d ** -0.5
    out, lse = H.run_prefill(q, k, v, s, l, scale, block=b)
    rb, rh, ri = H.all_rows(B, Hq, S)
    H.compare_prefill(q, k, v, out, lse, rb, rh, ri, s, l, scale, f"f32 blocks S{S} s{s} l{l} b{b}", block=b)


@pytest.mark.parametrize("B,Hq,S,s,l,b", [
    (1, 64, 700, 1, 2, 128),     # paper-sized blocks, several window edges inside workgroup tiles
    (1, 64, 300, 1, 7, 128),     # the paper's sizes on a sequence shorter than their live set
    (2, 16, 257, 2, 3, 20),      # block size that is no multiple of the key tile
    (1, 8, 700, 0, 2, 33),
    (1, 64, 131, 1, 1, 1),       # block of one token
    (1, 3, 150, 1, 2, 64),
])
def test_mla_bf16_prefill_blocks(gpu_device, B, Hq, S, s, l, b):
    q = _rand((B, S, Hq, 576), 11, torch.bfloat16, gpu_device)
    k = _rand((B, S, 1, 576), 12, torch.bfloat16, gpu_device)
    scale = 192 ** -0.5
    out, lse = H.run_prefill(q, k, k, s, l, scale, d_v=512, block=b)
    rb, rh, ri = H.all_rows(B, Hq, S)
    H.compare_prefill(q, k, k, out, lse, rb, rh, ri, s, l, scale, f"mla blocks B{B} Hq{Hq} S{S} s{s} l{l} b{b}", block=b)


@pytest.mark.parametrize("Hq,Hkv,S,s,l,b", [(4, 4, 1000, 1, 3, 128), (8, 2, 333, 1, 2, 50)])
def test_d128_bf16_prefill_blocks(gpu_device, Hq, Hkv, S, s, l, b):
    q = _rand((1, S, Hq, 128), 21, torch.bfloat16, gpu_device)
    k = _rand((1, S, Hkv, 128), 22, torch.bfloat16, gpu_device)
    v = _rand((1, S, Hkv, 128), 23, torch.bfloat16, gpu_device)
    scale = 128 ** -0.5
    out, lse = H.run_prefill(q, k, v, s, l, scale, block=b)
    rb, rh, ri = H.all_rows(1, Hq, S)
    H.compare_prefill(q, k, v, out, lse, rb, rh, ri, s, l, scale, f"d128 blocks Hq{Hq} Hkv{Hkv} S{S} s{s} l{l} b{b}", block=b)


@pytest.mark.parametrize("dtype,S,Hq,s,l,b", [
    (torch.float32, 1024, 1, 1, 2, 128),
    (torch.bfloat16, 1024, 2, 1, 3, 128),
    (torch.bfloat16, 700, 64, 1, 2, 96),
    (torch.bfloat16, 520, 5, 0, 2, 37),
])
def test_block_index_set_is_bit_exact(gpu_device, dtype, S, Hq, s, l, b):
    """Q = 0 and one-hot value columns: out[i, c] != 0 exactly where key j_c is live for query i, and
    lse = ln |live(i)|. Recovers the whole S x S mask of the kernel, d_v key columns per launch."""
    d_qk, d_v = (576, 512) if dtype == torch.bfloat16 else (64, 64)
    mask = np.zeros((S, S), dtype=bool)
    q = torch.zeros(1, S, Hq, d_qk, dtype=dtype, device=gpu_device)
    lse_row = None
    for j0 in range(0, S, d_v):
        kv = torch.zeros(1, S, 1, d_qk, dtype=dtype, device=gpu_device)
        n = min(d_v, S - j0)
        kv[0, j0 + torch.arange(n), 0, torch.arange(n)] = 1.0
        v = kv if dtype == torch.bfloat16 else kv[..., :d_v].contiguous()
        out, lse = H.run_prefill(q, kv, v, s, l, 1.0, d_v=d_v, block=b)
        mask[:, j0:j0 + n] = out[0, :, Hq - 1, :n].float().cpu().numpy() != 0.0
        lse_row = lse[0, Hq - 1].cpu().numpy()
    want = np.stack([oracle.live_mask_blocks(i, S, s, l, b).astype(bool) for i in range(S)])
    assert (mask == want).all(), f"index set differs at {np.argwhere(mask != want)[:5]}"
    np.testing.assert_allclose(lse_row, np.log(want.sum(1)), atol=1e-5)


@pytest.mark.parametrize("B,Hq,S_max,lens,s,l,b", [
    (3, 64, 1500, [1500, 1025, 1], 1, 7, 128),     # the paper's sizes; a query that opens a new block
    (4, 16, 1000, [999, 64, 65, 513], 0, 2, 50),
    (3, 5, 200, [0, 200, 17], 1, 1, 16),           # an empty cache among the batch
    (2, 64, 2500, [2500, 1777], 1, 3, 1),          # block of one token
])
def test_mla_bf16_decode_blocks(gpu_device, B, Hq, S_max, lens, s, l, b):
    q = _rand((B, Hq, 576), 41, torch.bfloat16, gpu_device)
    kc = _rand((B, S_max, 1, 576), 42, torch.bfloat16, gpu_device)
    for bi, L in enumerate(lens):
        kc[bi, L:] = float("nan")  # rows past the length must never be read
    seqlens = torch.tensor(lens, dtype=torch.int32, device=gpu_device)
    scale = 192 ** -0.5
    out, lse = H.run_decode(q, kc, kc, seqlens, s, l, scale, d_v=512, block=b)
    live = [bi for bi, L in enumerate(lens) if L > 0]
    rb = np.repeat(np.asarray(live, dtype=np.int64), Hq)
    rh = np.tile(np.arange(Hq, dtype=np.int64), len(live))
    H.compare_decode(q, kc, kc, seqlens, out, lse, rb, rh, s, l, scale, f"decode blocks lens{lens} s{s} l{l} b{b}", block=b)
    for bi, L in enumerate(lens):
        if L == 0:
            assert (out[bi] == 0).all() and torch.isneginf(lse[bi]).all()


def test_block_of_one_token_gives_the_bits_of_the_token_granular_entry_point(gpu_device):
    q = _rand((1, 400, 64, 576), 31, torch.bfloat16, gpu_device)
    k = _rand((1, 400, 1, 576), 32, torch.bfloat16, gpu_device)
    a = H.run_prefill(q, k, k, 16, 130, 0.07, d_v=512)
    c = H.run_prefill(q, k, k, 16, 130, 0.07, d_v=512, block=1)
    assert torch.equal(a[0].view(torch.int16), c[0].view(torch.int16))
    assert torch.equal(a[1].view(torch.int32), c[1].view(torch.int32))


# ---- the paper's sizes at the 128K shapes (sampled rows) ------------------------------------------

PAPER_S, PAPER_L, PAPER_B = 1, 7, 128


def test_paper_sizes_mla_prefill_128k(gpu_device):
    cfg = W.CFG3
    q, k, v = W.make_prefill_inputs(cfg, gpu_device)
    out, lse = H.run_prefill(q, k, v, PAPER_S, PAPER_L, cfg.scale, d_v=cfg.d_v, block=PAPER_B)
    # sample as for a token pattern with the same sink and the largest window, plus both ends of blocks
    like = replace(cfg, n_sink=PAPER_S * PAPER_B, window=PAPER_L * PAPER_B)
    rb, rh, ri = W.sample_rows(like, n_random=256, n_heads=4)
    extra = np.asarray([1023, 1024, 1151, 1152, 65535, 65536, 65663, 131071 - 127], dtype=np.int64)
    heads = np.unique(rh)
    rb = np.concatenate([rb, np.zeros(len(extra) * len(heads), dtype=np.int64)])
    rh = np.concatenate([rh, np.repeat(heads, len(extra))])
    ri = np.concatenate([ri, np.tile(extra, len(heads))])
    H.compare_prefill(q, k, v, out, lse, rb, rh, ri, PAPER_S, PAPER_L, cfg.scale, "cfg3 shape, s1 l7 b128", block=PAPER_B)


def test_paper_sizes_mla_decode_b64(gpu_device):
    cfg = W.CFG4
    q, kc, vc, seqlens = W.make_decode_inputs(cfg, gpu_device, poison_tail=True)
    out, lse = H.run_decode(q, kc, vc, seqlens, PAPER_S, PAPER_L, cfg.scale, d_v=cfg.d_v, block=PAPER_B)
    heads = np.asarray([0, 17, 32, 63], dtype=np.int64)
    rb = np.repeat(np.arange(cfg.B, dtype=np.int64), len(heads))
    rh = np.tile(heads, cfg.B)
    H.compare_decode(q, kc, vc, seqlens, out, lse, rb, rh, PAPER_S, PAPER_L, cfg.scale, "cfg4 shape, s1 l7 b128", block=PAPER_B)
    assert torch.isfinite(out.float()).all() and torch.isfinite(lse).all()
