"""GPU parity of the "extend" form (q_len new query tokens per sequence against its cache): every
query against the oracle at its position seqlens[b] - q_len + r, element by element."""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_23966_amd as loza
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _rand(shape, seed, dtype, device):
    g = torch.Generator(device=device).manual_seed(seed)
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32).to(dtype)


def _run(q, kc, vc, seqlens, pattern, scale, d_v, block=None):
    B, q_len, Hq, _ = q.shape
    out = torch.empty(B, q_len, Hq, d_v, dtype=torch.bfloat16, device=q.device)
    lse = torch.empty(B, Hq, q_len, dtype=torch.float32, device=q.device)
    if block is None:
        loza.loza_ssa_extend(q, kc, vc, seqlens, out, lse, pattern[0], pattern[1], scale)
    else:
        loza.loza_ssa_extend_blocks(q, kc, vc, seqlens, out, lse, pattern[0], pattern[1], block, scale)
    torch.cuda.synchronize()
    return out, lse


def _compare(q, kc, vc, lens, out, lse, pattern, scale, label, block=None):
    """All (b, r, h) whose position is >= 0 against the oracle; the others must be 0 / -inf."""
    B, q_len, Hq, _ = q.shape
    d_v = out.shape[3]
    rb, rr, rh = [], [], []
    for b, L in enumerate(lens):
        for r in range(q_len):
            if L - q_len + r >= 0:
                rb += [b] * Hq; rr += [r] * Hq; rh += list(range(Hq))
            else:
                assert (out[b, r] == 0).all(), f"{label}: query before the sequence start must give 0"
                assert torch.isneginf(lse[b, :, r]).all()
    rb, rr, rh = (np.asarray(x, dtype=np.int64) for x in (rb, rr, rh))
    ri = np.asarray(lens, dtype=np.int64)[rb] - q_len + rr
    dev = q.device
    tb, tr, th = (torch.as_tensor(x, device=dev) for x in (rb, rr, rh))
    q_rows = q[tb, tr, th].contiguous().cpu()
    varg = ("alias", d_v) if vc is kc else vc.cpu()
    w = oracle.INT64_MAX if pattern[1] is None else pattern[1]
    ref_out, ref_lse = oracle.ssa_rows(q_rows, kc.cpu(), varg, rb, rh, ri, Hq=Hq, n_sink=pattern[0], window=w, scale=scale,
                                       block=block)
    H._judge(out[tb, tr, th].double().cpu().numpy(), ref_out, lse[tb, th, tr].double().cpu().numpy(), ref_lse,
             torch.bfloat16, len(rb), label)


CASES = [
    # B, Hq, S_max, q_len, lens, n_sink, window, block
    (3, 64, 600, 4, [600, 257, 131], 128, 100, None),     # a few speculated tokens; one sequence around position 128
    (2, 64, 500, 37, [500, 300], 16, 64, None),           # a chunk that is no multiple of anything
    (3, 16, 400, 50, [400, 20, 0], 8, 30, None),          # a chunk longer than one cache, and an empty cache
    (2, 64, 1500, 130, [1500, 1100], 1, 7, 128),          # the paper's block pattern, chunk crossing blocks
    (1, 8, 700, 700, [700], 33, 95, None),                # the whole sequence as one chunk: a plain prefill
    (2, 64, 300, 5, [130, 127], 128, None, None),         # window = infinity; chunks around position 128
]


@pytest.mark.parametrize("B,Hq,S_max,q_len,lens,ns,win,block", CASES)
def test_mla_bf16_extend(gpu_device, B, Hq, S_max, q_len, lens, ns, win, block):
    q = _rand((B, q_len, Hq, 576), 71, torch.bfloat16, gpu_device)
    kc = _rand((B, S_max, 1, 576), 72, torch.bfloat16, gpu_device)
    for b, L in enumerate(lens):
        kc[b, L:] = float("nan")  # rows past the length must never be read
    seqlens = torch.tensor(lens, dtype=torch.int32, device=gpu_device)
    scale = 192 ** -0.5
    out, lse = _run(q, kc, kc, seqlens, (ns, win), scale, 512, block)
    _compare(q, kc, kc, lens, out, lse, (ns, win), scale, f"extend q{q_len} lens{lens} ns{ns} W{win} b{block}", block)


def test_d128_bf16_extend_grouped_heads(gpu_device):
    B, Hq, Hkv, S_max, q_len, lens, ns, win = 2, 8, 2, 900, 70, [900, 333], 32, 200
    q = _rand((B, q_len, Hq, 128), 81, torch.bfloat16, gpu_device)
    kc = _rand((B, S_max, Hkv, 128), 82, torch.bfloat16, gpu_device)
    vc = _rand((B, S_max, Hkv, 128), 83, torch.bfloat16, gpu_device)
    seqlens = torch.tensor(lens, dtype=torch.int32, device=gpu_device)
    scale = 128 ** -0.5
    out, lse = _run(q, kc, vc, seqlens, (ns, win), scale, 128)
    _compare(q, kc, vc, lens, out, lse, (ns, win), scale, "extend d128")


def test_whole_sequence_chunk_gives_the_bits_of_prefill(gpu_device):
    S, Hq = 450, 64
    q = _rand((1, S, Hq, 576), 91, torch.bfloat16, gpu_device)
    k = _rand((1, S, 1, 576), 92, torch.bfloat16, gpu_device)
    seqlens = torch.tensor([S], dtype=torch.int32, device=gpu_device)
    out_e, lse_e = _run(q, k, k, seqlens, (16, 130), 0.07, 512)
    out_p, lse_p = H.run_prefill(q, k, k, 16, 130, 0.07, d_v=512)
    assert torch.equal(out_e.view(torch.int16), out_p.view(torch.int16))
    assert torch.equal(lse_e.view(torch.int32), lse_p.view(torch.int32))


def test_single_token_chunk_agrees_with_decode(gpu_device):
    B, Hq, S_max, lens, ns, win = 3, 64, 3000, [3000, 1500, 400], 128, 1024
    q = _rand((B, 1, Hq, 576), 95, torch.bfloat16, gpu_device)
    kc = _rand((B, S_max, 1, 576), 96, torch.bfloat16, gpu_device)
    seqlens = torch.tensor(lens, dtype=torch.int32, device=gpu_device)
    scale = 192 ** -0.5
    out_e, lse_e = _run(q, kc, kc, seqlens, (ns, win), scale, 512)
    out_d, lse_d = H.run_decode(q[:, 0].contiguous(), kc, kc, seqlens, ns, win, scale, d_v=512)
    assert (out_e[:, 0].float() - out_d.float()).abs().max().item() <= 1.6e-2   # two independent bf16 roundings
    assert (lse_e[:, :, 0] - lse_d).abs().max().item() <= 1e-4


# ---- extend against a paged cache ------------------------------------------------------------------

def _run_paged(q, k_pages, v_pages, table, seqlens, pattern, scale, d_v, block=None):
    B, q_len, Hq, _ = q.shape
    out = torch.empty(B, q_len, Hq, d_v, dtype=torch.bfloat16, device=q.device)
    lse = torch.empty(B, Hq, q_len, dtype=torch.float32, device=q.device)
    if block is None:
        loza.loza_ssa_extend_paged(q, k_pages, v_pages, table, seqlens, out, lse, pattern[0], pattern[1], scale)
    else:
        loza.loza_ssa_extend_paged_blocks(q, k_pages, v_pages, table, seqlens, out, lse, pattern[0], pattern[1], block, scale)
    torch.cuda.synchronize()
    return out, lse


@pytest.mark.parametrize("B,Hq,S_max,q_len,lens,ns,win,page,block", [
    (3, 64, 640, 4, [600, 257, 131], 128, 100, 128, None),
    (2, 64, 512, 37, [500, 300], 16, 64, 32, None),
    (2, 64, 1536, 130, [1500, 1100], 1, 7, 128, 128),     # the paper's pattern, page = block
    (2, 16, 512, 50, [400, 20], 8, 30, 64, None),          # a chunk longer than one of the caches
])
def test_mla_bf16_extend_paged_equals_contiguous(gpu_device, B, Hq, S_max, q_len, lens, ns, win, page, block):
    from tests.test_gpu_parity_paged import _paginate
    q = _rand((B, q_len, Hq, 576), 71, torch.bfloat16, gpu_device)
    kc = _rand((B, S_max, 1, 576), 72, torch.bfloat16, gpu_device)
    for b, L in enumerate(lens):
        kc[b, L:] = float("nan")
    seqlens = torch.tensor(lens, dtype=torch.int32, device=gpu_device)
    scale = 192 ** -0.5
    pages, table = _paginate(kc, lens, page, seed=3)
    out_p, lse_p = _run_paged(q, pages, pages, table, seqlens, (ns, win), scale, 512, block)
    out_c, lse_c = _run(q, kc, kc, seqlens, (ns, win), scale, 512, block)
    assert torch.equal(out_p.view(torch.int16), out_c.view(torch.int16)), "paged and contiguous extend differ"
    assert torch.equal(lse_p.view(torch.int32), lse_c.view(torch.int32))
    _compare(q, kc, kc, lens, out_p, lse_p, (ns, win), scale, f"extend paged q{q_len} lens{lens} page{page} b{block}", block)
