"""Output buffers between guard zones: no entry point may write a byte outside the tensors it is given.

Every output (and the workspace) of a call sits inside one larger byte buffer, 256-byte aligned, with
4 KiB of a sentinel pattern in front of it and behind it; after the call the guard zones must still hold
the pattern and every element of the output must have been written (the outputs start as the pattern,
which no result can be: it reads as a NaN in bf16 and in fp32). Shapes are ragged on purpose (rows and
keys that are no multiple of any tile), where an unguarded tail store would land in the zone behind."""
import numpy as np
import pytest
import torch

import paper_2512_23966_amd as loza

pytestmark = pytest.mark.gpu

GUARD = 4096
PATTERN = 0xFF          # 0xFFFF is a bf16 NaN, 0xFFFFFFFF an fp32 NaN


class Guarded:
    """Tensors carved out of guarded byte buffers."""

    def __init__(self, device):
        self.device = device
        self.buffers = []

    def tensor(self, shape, dtype):
        n = int(np.prod(shape)) * torch.empty((), dtype=dtype).element_size()
        n_pad = (n + 255) // 256 * 256
        raw = torch.full((GUARD + n_pad + GUARD,), PATTERN, dtype=torch.uint8, device=self.device)
        t = raw[GUARD:GUARD + n].view(dtype).view(*shape)
        assert t.data_ptr() % 256 == 0 and t.is_contiguous()
        self.buffers.append((raw, n))
        return t

    def check(self, label):
        torch.cuda.synchronize()
        for raw, n in self.buffers:
            front, back = raw[:GUARD], raw[GUARD + n:]
            assert bool((front == PATTERN).all()), f"{label}: bytes in front of a buffer of {n} bytes were overwritten"
            assert bool((back == PATTERN).all()), f"{label}: bytes behind a buffer of {n} bytes were overwritten"


def _rand(shape, seed, device, dtype=torch.bfloat16):
    g = torch.Generator(device=device).manual_seed(seed)
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32).to(dtype)


def _all_written(t, label):
    assert not bool(torch.isnan(t.float()).any()), f"{label}: an element of an output was not written"


@pytest.mark.parametrize("S,Hq,Hkv,d_qk,d_v,alias", [(333, 64, 1, 576, 512, True), (1037, 8, 2, 128, 128, False), (97, 64, 1, 576, 512, True)])
def test_prefill_and_backward_stay_inside_their_buffers(gpu_device, S, Hq, Hkv, d_qk, d_v, alias):
    ns, win, scale = 16, 100, d_qk ** -0.5
    q = _rand((1, S, Hq, d_qk), 1, gpu_device)
    k = _rand((1, S, Hkv, d_qk), 2, gpu_device)
    v = k if alias else _rand((1, S, Hkv, d_v), 3, gpu_device)
    G = Guarded(gpu_device)
    out, lse = G.tensor((1, S, Hq, d_v), torch.bfloat16), G.tensor((1, Hq, S), torch.float32)
    loza.loza_ssa_prefill(q, k, v, out, lse, ns, win, scale)
    G.check(f"prefill S{S}")
    _all_written(out, "prefill out"); _all_written(lse, "prefill lse")
    dout = _rand(out.shape, 4, gpu_device)
    dq, dk = G.tensor(q.shape, torch.bfloat16), G.tensor(k.shape, torch.bfloat16)
    dv = None if alias else G.tensor(v.shape, torch.bfloat16)
    nb = loza.loza_ssa_backward_workspace_bytes(1, Hq, Hkv, S, d_qk, d_v, ns, win, alias)
    ws = G.tensor((max(nb, 16),), torch.uint8)
    loza.loza_ssa_backward(q, k, v, out, lse, dout, dq, dk, dv, ns, win, scale, ws)
    G.check(f"backward S{S}")
    _all_written(dq, "dq"); _all_written(dk, "dk")
    if dv is not None:
        _all_written(dv, "dv")


def test_prefill_f32_stays_inside_its_buffers(gpu_device):
    S, Hq, Hkv, d = 211, 6, 2, 72
    q, k, v = (_rand((1, S, h, d), s, gpu_device, torch.float32) for h, s in ((Hq, 1), (Hkv, 2), (Hkv, 3)))
    G = Guarded(gpu_device)
    out, lse = G.tensor((1, S, Hq, d), torch.float32), G.tensor((1, Hq, S), torch.float32)
    loza.loza_ssa_prefill_f32(q, k, v, out, lse, 5, 40, d ** -0.5)
    G.check("prefill f32")
    _all_written(out, "out"); _all_written(lse, "lse")


@pytest.mark.parametrize("paged", [False, True])
def test_decode_and_extend_stay_inside_their_buffers(gpu_device, paged):
    B, Hq, S_max, ns, win, scale = 5, 64, 1000, 128, 300, 192 ** -0.5
    lens = [1000, 1, 517, 0, 129]
    kc = _rand((B, S_max, 1, 576), 5, gpu_device)
    seqlens = torch.tensor(lens, dtype=torch.int32, device=gpu_device)
    G = Guarded(gpu_device)
    q = _rand((B, Hq, 576), 6, gpu_device)
    out, lse = G.tensor((B, Hq, 512), torch.bfloat16), G.tensor((B, Hq), torch.float32)
    nb = loza.loza_ssa_decode_workspace_bytes(B, Hq, 1, S_max, 512, ns, win)
    ws = G.tensor((max(nb, 16),), torch.uint8)
    q_len = 37
    qe = _rand((B, q_len, Hq, 576), 7, gpu_device)
    oute, lsee = G.tensor((B, q_len, Hq, 512), torch.bfloat16), G.tensor((B, Hq, q_len), torch.float32)
    if not paged:
        loza.loza_ssa_decode(q, kc, kc, seqlens, out, lse, ns, win, scale, ws)
        loza.loza_ssa_extend(qe, kc, kc, seqlens, oute, lsee, ns, win, scale)
    else:
        page = 128
        pages_per_seq = (S_max + page - 1) // page
        n_pages = B * pages_per_seq
        perm = torch.randperm(n_pages, generator=torch.Generator().manual_seed(3)).to(torch.int32)
        table = perm.view(B, pages_per_seq).to(gpu_device)
        pool = torch.zeros(n_pages, page, 1, 576, dtype=torch.bfloat16, device=gpu_device)
        for b in range(B):
            for pg in range(pages_per_seq):
                rows = kc[b, pg * page:(pg + 1) * page]
                pool[int(perm[b * pages_per_seq + pg]), :rows.shape[0]] = rows
        loza.loza_ssa_decode_paged(q, pool, pool, table, seqlens, out, lse, ns, win, scale, ws)
        loza.loza_ssa_extend_paged(qe, pool, pool, table, seqlens, oute, lsee, ns, win, scale)
    G.check(f"decode / extend, paged={paged}")
    for t, name in ((out, "decode out"), (oute, "extend out")):
        _all_written(t, name)
    # (a log-sum-exp of -inf is a legal value for an empty cache or a query before the sequence start; NaN is not)
    assert not bool(torch.isnan(lse).any()) and not bool(torch.isnan(lsee).any())
