"""GPU parity of the paged-cache decode: the same rows scattered over physical pages behind a block
table must give the bits of the contiguous-cache decode, and both must match the oracle (which
reads the contiguous rows: paging is storage, not arithmetic)."""
import numpy as np
import pytest
import torch

import paper_2512_23966_amd as loza
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _rand(shape, seed, dtype, device):
    g = torch.Generator(device=device).manual_seed(seed)
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32).to(dtype)


def _paginate(cache, lens, page_size, seed, spare_pages=3):
    """Scatter the valid rows of a contiguous cache [B, S_max, Hkv, d] over shuffled physical pages.
    Returns (pages [num_pages, page_size, Hkv, d], block_table [B, max_pages] int32). Pages and table
    entries nobody may read are poisoned (NaN rows, out-of-range page numbers)."""
    B, S_max, Hkv, d = cache.shape
    max_pages = (S_max + page_size - 1) // page_size
    need = [(L + page_size - 1) // page_size for L in lens]
    num_pages = sum(need) + spare_pages
    rng = np.random.default_rng(seed)
    phys = rng.permutation(num_pages)
    pages = torch.full((num_pages, page_size, Hkv, d), float("nan"), dtype=cache.dtype, device=cache.device)
    table = np.full((B, max_pages), 2 ** 30, dtype=np.int32)   # never to be used
    table[:, ::2] = -7
    nxt = 0
    for b, L in enumerate(lens):
        for lp in range(need[b]):
            pid = int(phys[nxt]); nxt += 1
            table[b, lp] = pid
            r0, r1 = lp * page_size, min((lp + 1) * page_size, L)
            pages[pid, : r1 - r0] = cache[b, r0:r1]
    return pages, torch.as_tensor(table, device=cache.device)


def _run_paged(q, k_pages, v_pages, table, seqlens, ns, win, scale, d_v, block=None):
    B, Hq, _ = q.shape
    _, page_size, Hkv, _ = k_pages.shape
    S_cap = table.shape[1] * page_size
    out = torch.empty(B, Hq, d_v, dtype=torch.bfloat16, device=q.device)
    lse = torch.empty(B, Hq, dtype=torch.float32, device=q.device)
    if block is None:
        nb = loza.loza_ssa_decode_workspace_bytes(B, Hq, Hkv, S_cap, d_v, ns, win)
        ws = torch.empty(max(nb, 16), dtype=torch.uint8, device=q.device)
        loza.loza_ssa_decode_paged(q, k_pages, v_pages, table, seqlens, out, lse, ns, win, scale, ws)
    else:
        nb = loza.loza_ssa_decode_workspace_bytes(B, Hq, Hkv, S_cap, d_v, ns * block, None if win is None else win * block)
        ws = torch.empty(max(nb, 16), dtype=torch.uint8, device=q.device)
        loza.loza_ssa_decode_paged_blocks(q, k_pages, v_pages, table, seqlens, out, lse, ns, win, block, scale, ws)
    torch.cuda.synchronize()
    return out, lse


CASES = [
    # B, Hq, S_max, lens, n_sink, window, page_size, block (None: token-granular)
    (3, 64, 4096, [4096, 2049, 1], 128, 1024, 128, None),    # paper-sized pages; a one-row sequence
    (2, 64, 3000, [3000, 1777], 128, 1024, 32, None),        # a page per key tile
    (4, 16, 1024, [999, 64, 65, 513], 0, 70, 256, None),     # pages larger than most windows
    (3, 64, 2048, [2048, 1025, 130], 1, 7, 128, 128),        # the paper's block pattern, page = block
    (3, 5, 512, [0, 200, 17], 4, 9, 64, None),               # an empty cache; short ones (direct path)
    (1, 64, 768, [700], 7, None, 128, None),                 # window = infinity: every page is read
]


@pytest.mark.parametrize("B,Hq,S_max,lens,ns,win,page,block", CASES)
def test_mla_bf16_decode_paged(gpu_device, B, Hq, S_max, lens, ns, win, page, block):
    q = _rand((B, Hq, 576), 41, torch.bfloat16, gpu_device)
    kc = _rand((B, S_max, 1, 576), 42, torch.bfloat16, gpu_device)
    for b, L in enumerate(lens):
        kc[b, L:] = float("nan")
    seqlens = torch.tensor(lens, dtype=torch.int32, device=gpu_device)
    scale = 192 ** -0.5
    pages, table = _paginate(kc, lens, page, seed=5)
    out_p, lse_p = _run_paged(q, pages, pages, table, seqlens, ns, win, scale, 512, block)
    out_c, lse_c = H.run_decode(q, kc, kc, seqlens, ns, win, scale, d_v=512, block=block)
    # (the same bits as long as both calls cut the keys into the same number of splits, which the
    # cases arrange: where the pattern reaches the whole cache, its capacity is a multiple of the page)
    assert torch.equal(out_p.view(torch.int16), out_c.view(torch.int16)), "paged and contiguous decode differ"
    assert torch.equal(lse_p.view(torch.int32), lse_c.view(torch.int32))
    live = [b for b, L in enumerate(lens) if L > 0]
    rb = np.repeat(np.asarray(live, dtype=np.int64), Hq)
    rh = np.tile(np.arange(Hq, dtype=np.int64), len(live))
    H.compare_decode(q, kc, kc, seqlens, out_p, lse_p, rb, rh, ns, win, scale,
                     f"paged decode lens{lens} ns{ns} W{win} page{page} block{block}", block=block)
    for b, L in enumerate(lens):
        if L == 0:
            assert (out_p[b] == 0).all() and torch.isneginf(lse_p[b]).all()


def test_d128_bf16_decode_paged_separate_values(gpu_device):
    B, Hq, Hkv, S_max, lens, ns, win, page = 3, 8, 2, 600, [600, 129, 40], 32, 200, 64
    q = _rand((B, Hq, 128), 51, torch.bfloat16, gpu_device)
    kc = _rand((B, S_max, Hkv, 128), 52, torch.bfloat16, gpu_device)
    vc = _rand((B, S_max, Hkv, 128), 53, torch.bfloat16, gpu_device)
    seqlens = torch.tensor(lens, dtype=torch.int32, device=gpu_device)
    scale = 128 ** -0.5
    k_pages, table = _paginate(kc, lens, page, seed=9)
    v_pages, table_v = _paginate(vc, lens, page, seed=9)
    assert torch.equal(table, table_v)
    out_p, lse_p = _run_paged(q, k_pages, v_pages, table, seqlens, ns, win, scale, 128)
    rb = np.repeat(np.arange(B, dtype=np.int64), Hq)
    rh = np.tile(np.arange(Hq, dtype=np.int64), B)
    H.compare_decode(q, kc, vc, seqlens, out_p, lse_p, rb, rh, ns, win, scale, "paged decode d128")


def test_paged_decode_at_the_benchmark_shape(gpu_device):
    """64 sequences with cache lengths in [65536, 262144], pages of 128 rows shuffled over one pool."""
    from paper_2512_23966_amd import workloads as W
    cfg = W.CFG4
    q, kc, vc, seqlens = W.make_decode_inputs(cfg, gpu_device)
    lens = seqlens.cpu().numpy().astype(np.int64)
    page = 128
    max_pages = cfg.S_max // page
    # The pool is the contiguous cache itself seen as pages of 128 rows (2048 per sequence). To make
    # the table matter, the physical pages of the two most recent logical pages of every sequence
    # are swapped in memory and in the table; afterwards the swap is undone for the reference run.
    pool = kc.view(cfg.B * max_pages, page, 1, cfg.d_qk)
    table = torch.arange(cfg.B * max_pages, dtype=torch.int32, device=gpu_device).view(cfg.B, max_pages).clone()
    for b in range(cfg.B):
        last = int((lens[b] - 1) // page)
        a_, c_ = b * max_pages + last, b * max_pages + last - 1
        tmp = pool[a_].clone(); pool[a_] = pool[c_]; pool[c_] = tmp
        table[b, last], table[b, last - 1] = c_, a_
    out_p, lse_p = _run_paged(q, pool, pool, table, seqlens, cfg.n_sink, cfg.window, cfg.scale, cfg.d_v)
    # undo the swap: the contiguous view is the reference layout again
    for b in range(cfg.B):
        last = int((lens[b] - 1) // page)
        a_, c_ = b * max_pages + last, b * max_pages + last - 1
        tmp = pool[a_].clone(); pool[a_] = pool[c_]; pool[c_] = tmp
    out_c, lse_c = H.run_decode(q, kc, vc, seqlens, cfg.n_sink, cfg.window, cfg.scale, d_v=cfg.d_v)
    diff = (out_p.view(torch.int16) != out_c.view(torch.int16)).nonzero()
    assert diff.numel() == 0, (f"paged and contiguous decode differ in {diff.shape[0]} elements; sequences "
                               f"{sorted(set(diff[:, 0].tolist()))[:8]}, heads {sorted(set(diff[:, 1].tolist()))[:8]}, columns "
                               f"{sorted(set(diff[:, 2].tolist()))[:8]}; max |difference| {(out_p.float() - out_c.float()).abs().max().item():.3e}")
    assert torch.equal(lse_p.view(torch.int32), lse_c.view(torch.int32))
    heads = np.asarray([0, 31, 63], dtype=np.int64)
    rb = np.repeat(np.arange(cfg.B, dtype=np.int64), len(heads))
    rh = np.tile(heads, cfg.B)
    H.compare_decode(q, kc, vc, seqlens, out_p, lse_p, rb, rh, cfg.n_sink, cfg.window, cfg.scale, "paged cfg4")
