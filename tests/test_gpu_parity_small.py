"""GPU parity, small sizes: the HIP path against the fp64 oracle on every output element.

Sizes are chosen so the oracle finishes in seconds while the workload still spans several
workgroup tiles, both kinds of edge tile (causal diagonal, window trailing edge), the sink edge,
the sink/window overlap region and a ragged last tile.
"""
import numpy as np
import pytest
import torch

import paper_2512_23966_amd as loza
from paper_2512_23966_amd import workloads as W
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _rand(shape, seed, dtype, device):
    g = torch.Generator(device=device).manual_seed(seed)
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32).to(dtype)


def test_cfg1_tiny_fp32_prefill_full_parity(gpu_device):
    cfg = W.CFG1
    q, k, v = W.make_prefill_inputs(cfg, gpu_device)
    out, lse = H.run_prefill(q, k, v, cfg.n_sink, cfg.window, cfg.scale)
    rb, rh, ri = H.all_rows(cfg.B, cfg.Hq, cfg.S)
    H.compare_prefill(q, k, v, out, lse, rb, rh, ri, cfg.n_sink, cfg.window, cfg.scale, cfg.name)


@pytest.mark.parametrize("B,Hq,Hkv,S,d_qk,d_v,alias,ns,win", [
    (2, 3, 1, 97, 40, 24, False, 5, 11),
    (1, 4, 2, 130, 64, 64, False, 0, 1),
    (1, 2, 2, 70, 256, 256, False, 9, None),
    (1, 6, 3, 65, 96, 32, True, 70, 3),
])
def test_fp32_prefill_shapes(gpu_device, B, Hq, Hkv, S, d_qk, d_v, alias, ns, win):
    q = _rand((B, S, Hq, d_qk), 1, torch.float32, gpu_device)
    k = _rand((B, S, Hkv, d_qk), 2, torch.float32, gpu_device)
    v = k if alias else _rand((B, S, Hkv, d_v), 3, torch.float32, gpu_device)
    scale = d_qk ** -0.5  # unit-variance scores, as in the tiny configuration the 1e-5 bound is stated for
    out, lse = H.run_prefill(q, k, v, ns, win, scale, d_v=d_v)
    rb, rh, ri = H.all_rows(B, Hq, S)
    H.compare_prefill(q, k, v, out, lse, rb, rh, ri, ns, win, scale, f"f32 B{B} Hq{Hq} Hkv{Hkv} S{S} ns{ns} W{win}")


MLA_CASES = [
    # B, Hq, S, n_sink, window
    (1, 64, 300, 128, 100),     # 64 heads share the latent; sink edge inside a tile; ragged tail
    (1, 64, 131, 0, 1),         # no sink, window of the query alone
    (2, 16, 257, 40, 64),       # 8 positions per workgroup tile; batch of two
    (1, 64, 96, 128, 8192),     # S < n_sink: everything is causal prefix
    (1, 8, 700, 33, 95),        # 16 positions per tile; odd sizes
    (1, 64, 200, 5, None),      # window = infinity (full causal attention)
    (1, 3, 150, 7, 20),         # head count that does not divide the tile
]


@pytest.mark.parametrize("B,Hq,S,ns,win", MLA_CASES)
def test_mla_bf16_prefill_small(gpu_device, B, Hq, S, ns, win):
    q = _rand((B, S, Hq, 576), 11, torch.bfloat16, gpu_device)
    k = _rand((B, S, 1, 576), 12, torch.bfloat16, gpu_device)
    scale = 192 ** -0.5
    out, lse = H.run_prefill(q, k, k, ns, win, scale, d_v=512)
    rb, rh, ri = H.all_rows(B, Hq, S)
    H.compare_prefill(q, k, k, out, lse, rb, rh, ri, ns, win, scale, f"mla B{B} Hq{Hq} S{S} ns{ns} W{win}")


MHA_CASES = [
    # B, Hq, Hkv, S, n_sink, window, alias
    (1, 4, 4, 1000, 128, 300, False),   # several row tiles per head, window edge tiles, ragged tail
    (2, 8, 2, 333, 17, 64, False),      # grouped heads: 4 query heads per kv head
    (1, 2, 2, 129, 0, 5, False),
    (1, 4, 1, 260, 64, 77, True),       # values alias the keys
    (1, 2, 2, 513, 600, 4, False),      # n_sink > S
    (1, 1, 1, 400, 3, None, False),     # full attention
]


@pytest.mark.parametrize("B,Hq,Hkv,S,ns,win,alias", MHA_CASES)
def test_d128_bf16_prefill_small(gpu_device, B, Hq, Hkv, S, ns, win, alias):
    q = _rand((B, S, Hq, 128), 21, torch.bfloat16, gpu_device)
    k = _rand((B, S, Hkv, 128), 22, torch.bfloat16, gpu_device)
    v = k if alias else _rand((B, S, Hkv, 128), 23, torch.bfloat16, gpu_device)
    scale = 128 ** -0.5
    out, lse = H.run_prefill(q, k, v, ns, win, scale, d_v=128)
    rb, rh, ri = H.all_rows(B, Hq, S)
    H.compare_prefill(q, k, v, out, lse, rb, rh, ri, ns, win, scale, f"d128 B{B} Hq{Hq} Hkv{Hkv} S{S} ns{ns} W{win}")


def _probe_live_mask(gpu_device, S, Hq, ns, win, dtype):
    """Read the kernel's index set back: with Q = 0 every live key gets weight 1/|live(i)|, and with
    V[j, c] = 1 iff j == j_c the output column c is non-zero exactly when key j_c is live."""
    d_qk, d_v = (576, 512) if dtype == torch.bfloat16 else (64, 64)
    mask = np.zeros((S, S), dtype=bool)
    lse_all = None
    q = torch.zeros(1, S, Hq, d_qk, dtype=dtype, device=gpu_device)
    for j0 in range(0, S, d_v):
        kv = torch.zeros(1, S, 1, d_qk, dtype=dtype, device=gpu_device)
        n = min(d_v, S - j0)
        kv[0, j0 + torch.arange(n), 0, torch.arange(n)] = 1.0
        if dtype == torch.bfloat16:
            out, lse = H.run_prefill(q, kv, kv, ns, win, 1.0, d_v=d_v)
        else:
            out, lse = H.run_prefill(q, kv, kv[..., :d_v].contiguous(), ns, win, 1.0, d_v=d_v)
        o = out[0, :, Hq - 1, :n].float().cpu().numpy()
        mask[:, j0:j0 + n] = o != 0.0
        lse_all = lse[0, Hq - 1].cpu().numpy()
    return mask, lse_all


@pytest.mark.parametrize("dtype,S,Hq,ns,win", [
    (torch.float32, 1024, 1, 64, 256),       # the tiny configuration's full 1024 x 1024 mask
    (torch.bfloat16, 1024, 2, 64, 256),
    (torch.bfloat16, 700, 64, 128, 200),
    (torch.bfloat16, 520, 5, 0, 37),
])
def test_index_set_is_bit_exact(gpu_device, dtype, S, Hq, ns, win):
    import oracle
    mask, lse = _probe_live_mask(gpu_device, S, Hq, ns, win, dtype)
    want = np.stack([oracle.live_mask(i, S, ns, win).astype(bool) for i in range(S)])
    assert (mask == want).all(), f"index set differs at {np.argwhere(mask != want)[:5]}"
    np.testing.assert_allclose(lse, np.log(want.sum(1)), atol=1e-5)


def test_prefill_is_deterministic(gpu_device):
    q = _rand((1, 500, 64, 576), 31, torch.bfloat16, gpu_device)
    k = _rand((1, 500, 1, 576), 32, torch.bfloat16, gpu_device)
    a = H.run_prefill(q, k, k, 16, 130, 0.07, d_v=512)
    b = H.run_prefill(q, k, k, 16, 130, 0.07, d_v=512)
    assert torch.equal(a[0].view(torch.int16), b[0].view(torch.int16))
    assert torch.equal(a[1].view(torch.int32), b[1].view(torch.int32))


# ------------------------------------------------------------------ decode ------------------

DECODE_CASES = [
    # B, Hq, S_max, lens, n_sink, window
    (3, 64, 400, [400, 257, 1], 128, 100),
    (2, 64, 300, [90, 300], 128, 8192),          # shorter than the sink: plain causal prefix
    (4, 16, 1000, [999, 64, 65, 513], 0, 70),
    (2, 64, 2500, [2500, 1777], 128, 1024),      # several key tiles per split
    (1, 64, 333, [333], 7, None),                # window = infinity
    (3, 5, 200, [0, 200, 17], 4, 9),             # an empty cache among the batch
]


@pytest.mark.parametrize("B,Hq,S_max,lens,ns,win", DECODE_CASES)
def test_mla_bf16_decode_small(gpu_device, B, Hq, S_max, lens, ns, win):
    q = _rand((B, Hq, 576), 41, torch.bfloat16, gpu_device)
    kc = _rand((B, S_max, 1, 576), 42, torch.bfloat16, gpu_device)
    for b, L in enumerate(lens):
        kc[b, L:] = float("nan")  # rows past the length must never be read
    seqlens = torch.tensor(lens, dtype=torch.int32, device=gpu_device)
    scale = 192 ** -0.5
    out, lse = H.run_decode(q, kc, kc, seqlens, ns, win, scale, d_v=512)
    live = [b for b, L in enumerate(lens) if L > 0]
    rb = np.repeat(np.asarray(live, dtype=np.int64), Hq)
    rh = np.tile(np.arange(Hq, dtype=np.int64), len(live))
    H.compare_decode(q, kc, kc, seqlens, out, lse, rb, rh, ns, win, scale, f"decode B{B} Hq{Hq} lens{lens} ns{ns} W{win}")
    for b, L in enumerate(lens):
        if L == 0:
            assert (out[b] == 0).all() and torch.isneginf(lse[b]).all()


@pytest.mark.parametrize("Hq,Hkv,alias", [(8, 2, False), (4, 4, True)])
def test_d128_bf16_decode_small(gpu_device, Hq, Hkv, alias):
    B, S_max, lens, ns, win = 3, 600, [600, 129, 40], 32, 200
    q = _rand((B, Hq, 128), 51, torch.bfloat16, gpu_device)
    kc = _rand((B, S_max, Hkv, 128), 52, torch.bfloat16, gpu_device)
    vc = kc if alias else _rand((B, S_max, Hkv, 128), 53, torch.bfloat16, gpu_device)
    seqlens = torch.tensor(lens, dtype=torch.int32, device=gpu_device)
    scale = 128 ** -0.5
    out, lse = H.run_decode(q, kc, vc, seqlens, ns, win, scale, d_v=128)
    rb = np.repeat(np.arange(B, dtype=np.int64), Hq)
    rh = np.tile(np.arange(Hq, dtype=np.int64), B)
    H.compare_decode(q, kc, vc, seqlens, out, lse, rb, rh, ns, win, scale, f"decode d128 Hq{Hq} Hkv{Hkv}")


def test_decode_equals_last_prefill_row_and_split_count_does_not_matter(gpu_device, monkeypatch):
    S, Hq, ns, win, scale = 3000, 64, 128, 1500, 192 ** -0.5
    q = _rand((1, S, Hq, 576), 61, torch.bfloat16, gpu_device)
    k = _rand((1, S, 1, 576), 62, torch.bfloat16, gpu_device)
    out_p, lse_p = H.run_prefill(q, k, k, ns, win, scale, d_v=512)
    seqlens = torch.tensor([S], dtype=torch.int32, device=gpu_device)
    qd = q[:, S - 1].contiguous()
    results = []
    for splits in ("1", "3", "7", "26"):
        monkeypatch.setenv("LOZA_DECODE_SPLITS", splits)
        out_d, lse_d = H.run_decode(qd, k, k, seqlens, ns, win, scale, d_v=512)
        results.append((out_d.float(), lse_d))
        assert (out_d.float() - out_p[:, S - 1].float()).abs().max().item() <= 2e-2  # two bf16 roundings
        assert (lse_d - lse_p[:, :, S - 1]).abs().max().item() <= 1e-4
    for o, l in results[1:]:
        assert (o - results[0][0]).abs().max().item() <= 1.6e-2
        assert (l - results[0][1]).abs().max().item() <= 1e-4


def test_mla_shape_with_two_latent_heads(gpu_device):
    """The wide shape with Hkv = 2 (rows of the cache are strided by two heads): prefill and decode."""
    B, S, Hq, Hkv, ns, win = 1, 300, 8, 2, 16, 70
    q = _rand((B, S, Hq, 576), 201, torch.bfloat16, gpu_device)
    k = _rand((B, S, Hkv, 576), 202, torch.bfloat16, gpu_device)
    scale = 192 ** -0.5
    out, lse = H.run_prefill(q, k, k, ns, win, scale, d_v=512)
    rb, rh, ri = H.all_rows(B, Hq, S)
    H.compare_prefill(q, k, k, out, lse, rb, rh, ri, ns, win, scale, "mla Hkv2 prefill")
    lens = [300, 180]
    qd = _rand((2, Hq, 576), 203, torch.bfloat16, gpu_device)
    kc = _rand((2, S, Hkv, 576), 204, torch.bfloat16, gpu_device)
    seqlens = torch.tensor(lens, dtype=torch.int32, device=gpu_device)
    out_d, lse_d = H.run_decode(qd, kc, kc, seqlens, ns, win, scale, d_v=512)
    rb = np.repeat(np.arange(2, dtype=np.int64), Hq)
    rh = np.tile(np.arange(Hq, dtype=np.int64), 2)
    H.compare_decode(qd, kc, kc, seqlens, out_d, lse_d, rb, rh, ns, win, scale, "mla Hkv2 decode")


def test_calls_run_on_the_stream_they_are_given(gpu_device):
    """Work queued on a side stream behind a long-running kernel must not be visible before that
    stream is waited for, and must be complete after: the launches go where the caller says."""
    q = _rand((1, 600, 64, 576), 211, torch.bfloat16, gpu_device)
    k = _rand((1, 600, 1, 576), 212, torch.bfloat16, gpu_device)
    ref_out, ref_lse = H.run_prefill(q, k, k, 16, 130, 0.07, d_v=512)
    side = torch.cuda.Stream(device=gpu_device)
    out = torch.zeros_like(ref_out)
    lse = torch.zeros_like(ref_lse)
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        loza.loza_ssa_prefill(q, k, k, out, lse, 16, 130, 0.07)           # picks up the current (side) stream
    loza.loza_ssa_prefill(q, k, k, out, lse, 16, 130, 0.07, stream=side)  # and an explicit one
    side.synchronize()
    assert torch.equal(out.view(torch.int16), ref_out.view(torch.int16))
    assert torch.equal(lse.view(torch.int32), ref_lse.view(torch.int32))


def test_decode_length_beyond_the_cache_is_cut_to_it(gpu_device):
    B, Hq, S_max, ns, win = 2, 64, 500, 16, 200
    q = _rand((B, Hq, 576), 221, torch.bfloat16, gpu_device)
    kc = _rand((B, S_max, 1, 576), 222, torch.bfloat16, gpu_device)
    scale = 192 ** -0.5
    exact = torch.tensor([S_max, S_max], dtype=torch.int32, device=gpu_device)
    beyond = torch.tensor([S_max + 100, 2 ** 31 - 1], dtype=torch.int32, device=gpu_device)
    a = H.run_decode(q, kc, kc, exact, ns, win, scale, d_v=512)
    c = H.run_decode(q, kc, kc, beyond, ns, win, scale, d_v=512)
    assert torch.equal(a[0].view(torch.int16), c[0].view(torch.int16))
    assert torch.equal(a[1].view(torch.int32), c[1].view(torch.int32))
