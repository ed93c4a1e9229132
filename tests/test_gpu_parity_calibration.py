"""GPU parity of the calibration forward (Architecture section, Eq. 3): alpha * O + (1 - alpha) * O'
against the oracle's blend of its two attentions, element by element at small sizes and on sampled
rows of the 32K and 128K shapes."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import oracle
import paper_2512_23966_amd as loza
from paper_2512_23966_amd import workloads as W
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _rand(shape, seed, dtype, device):
    g = torch.Generator(device=device).manual_seed(seed)
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32).to(dtype)


def _run(q, k, v, s, l, b, alpha, scale, d_v, want_parts=True):
    B, S, Hq, _ = q.shape
    dev = q.device
    out = torch.empty(B, S, Hq, d_v, dtype=torch.bfloat16, device=dev)
    o_full = torch.empty_like(out) if want_parts else None
    o_sparse = torch.empty_like(out) if want_parts else None
    lse_f = torch.empty(B, Hq, S, dtype=torch.float32, device=dev)
    lse_s = torch.empty(B, Hq, S, dtype=torch.float32, device=dev)
    ws = torch.empty(loza.loza_ssa_calibration_workspace_bytes(B, Hq, S, d_v), dtype=torch.uint8, device=dev)
    loza.loza_ssa_prefill_calibration_blocks(q, k, v, out, o_full, o_sparse, lse_f, lse_s, s, l, b, alpha, scale, ws)
    torch.cuda.synchronize()
    return out, o_full, o_sparse, lse_f, lse_s


def _compare(q, k, v, res, rb, rh, ri, s, l, b, alpha, scale, label):
    out, o_full, o_sparse, lse_f, lse_s = res
    dev = q.device
    idx = (torch.as_tensor(rb, device=dev), torch.as_tensor(ri, device=dev), torch.as_tensor(rh, device=dev))
    lidx = (torch.as_tensor(rb, device=dev), torch.as_tensor(rh, device=dev), torch.as_tensor(ri, device=dev))
    q_rows = q[idx].contiguous().cpu()
    varg = ("alias", out.shape[3]) if v is k else v.cpu()
    ref, ref_f, ref_s, rl_f, rl_s = oracle.calibration_rows(q_rows, k.cpu(), varg, rb, rh, ri, Hq=q.shape[2], sink_blocks=s,
                                                            local_blocks=l, block=b, alpha=alpha, scale=scale)
    H._judge(out[idx].double().cpu().numpy(), ref, lse_f[lidx].double().cpu().numpy(), rl_f, torch.bfloat16, len(rb), label + " blend/lse_full")
    if o_full is not None:
        H._judge(o_full[idx].double().cpu().numpy(), ref_f, lse_s[lidx].double().cpu().numpy(), rl_s, torch.bfloat16, len(rb), label + " O/lse_sparse")
        H._judge(o_sparse[idx].double().cpu().numpy(), ref_s, lse_s[lidx].double().cpu().numpy(), rl_s, torch.bfloat16, len(rb), label + " O'")


@pytest.mark.parametrize("B,Hq,S,s,l,b,alpha", [
    (1, 64, 700, 1, 2, 128, 0.3),
    (2, 16, 257, 2, 3, 20, 0.9),
    (1, 8, 500, 4, 50, 1, 0.5),      # token-granular through block = 1
    (1, 64, 300, 1, 7, 128, 0.0),    # alpha = 0: the sparse output itself
    (1, 3, 150, 1, 2, 64, 1.0),      # alpha = 1: full attention itself
])
def test_mla_bf16_calibration_small(gpu_device, B, Hq, S, s, l, b, alpha):
    q = _rand((B, S, Hq, 576), 11, torch.bfloat16, gpu_device)
    k = _rand((B, S, 1, 576), 12, torch.bfloat16, gpu_device)
    scale = 192 ** -0.5
    res = _run(q, k, k, s, l, b, alpha, scale, 512)
    rb, rh, ri = H.all_rows(B, Hq, S)
    _compare(q, k, k, res, rb, rh, ri, s, l, b, alpha, scale, f"calib mla S{S} s{s} l{l} b{b} a{alpha}")
    out, o_full, o_sparse = res[0], res[1], res[2]
    if alpha == 0.0:
        assert torch.equal(out.view(torch.int16), o_sparse.view(torch.int16))
    if alpha == 1.0:
        assert torch.equal(out.view(torch.int16), o_full.view(torch.int16))


def test_d128_bf16_calibration_small(gpu_device):
    B, Hq, Hkv, S, s, l, b, alpha = 1, 8, 2, 600, 1, 2, 64, 0.6
    q = _rand((B, S, Hq, 128), 21, torch.bfloat16, gpu_device)
    k = _rand((B, S, Hkv, 128), 22, torch.bfloat16, gpu_device)
    v = _rand((B, S, Hkv, 128), 23, torch.bfloat16, gpu_device)
    scale = 128 ** -0.5
    res = _run(q, k, v, s, l, b, alpha, scale, 128)
    rb, rh, ri = H.all_rows(B, Hq, S)
    _compare(q, k, v, res, rb, rh, ri, s, l, b, alpha, scale, "calib d128")


def test_calibration_parts_equal_the_plain_entry_points(gpu_device):
    """O and O' written by the calibration call are the bits of the two plain prefill calls."""
    q = _rand((1, 400, 64, 576), 31, torch.bfloat16, gpu_device)
    k = _rand((1, 400, 1, 576), 32, torch.bfloat16, gpu_device)
    out, o_full, o_sparse, lse_f, lse_s = _run(q, k, k, 1, 2, 64, 0.5, 0.07, 512)
    full = H.run_prefill(q, k, k, 0, None, 0.07, d_v=512)
    sparse = H.run_prefill(q, k, k, 1, 2, 0.07, d_v=512, block=64)
    assert torch.equal(o_full.view(torch.int16), full[0].view(torch.int16))
    assert torch.equal(o_sparse.view(torch.int16), sparse[0].view(torch.int16))
    assert torch.equal(lse_f.view(torch.int32), full[1].view(torch.int32))
    assert torch.equal(lse_s.view(torch.int32), sparse[1].view(torch.int32))


def test_calibration_paper_sizes_mla_32k(gpu_device):
    """The MLA shape at 32K tokens with the paper's pattern (1 sink + 7 local blocks of 128), alpha = 0.5."""
    cfg = replace(W.CFG3, S=32768, name="mla_32k")
    q, k, v = W.make_prefill_inputs(cfg, gpu_device)
    res = _run(q, k, v, 1, 7, 128, 0.5, cfg.scale, cfg.d_v, want_parts=False)
    like = replace(cfg, n_sink=128, window=896)
    rb, rh, ri = W.sample_rows(like, n_random=96, n_heads=3)
    _compare(q, k, v, res, rb, rh, ri, 1, 7, 128, 0.5, cfg.scale, "calib mla 32K s1 l7 b128")


@pytest.mark.parametrize("shape,seed", [((8,), 1), ((3, 7, 2, 8), 2), ((1, 700, 8, 128), 3), ((2, 4096, 64, 8 * 9), 4)])
def test_alpha_gradient(gpu_device, shape, seed):
    """d(alpha) = sum(dout * (O - O')) on synthetic bf16 tensors (one element up to 4.7 million elements per
    workgroup partial), against the oracle's float64 sum; the only rounding is the final one to fp32."""
    dout, o_full, o_sparse = (_rand(shape, 100 * seed + i, torch.bfloat16, gpu_device) for i in range(3))
    dalpha = torch.full((1,), float("nan"), dtype=torch.float32, device=gpu_device)
    n = dout.numel()
    ws = torch.empty(loza.loza_ssa_calibration_alpha_grad_workspace_bytes(n), dtype=torch.uint8, device=gpu_device)
    loza.loza_ssa_calibration_alpha_grad(dout, o_full, o_sparse, dalpha, ws)
    torch.cuda.synchronize()
    ref = oracle.calibration_alpha_grad(dout, o_full, o_sparse)
    got = float(dalpha.item())
    scale = float(np.sqrt(n)) * 2.0   # size of a sum of n products of N(0,1) values times N(0,2)
    print(f"[parity] alpha gradient n={n}: got {got:.9g} ref {ref:.9g}", flush=True)
    assert abs(got - ref) <= 2.0 ** -23 * max(abs(ref), 1e-30) + 1e-12 * scale
    again = torch.empty_like(dalpha)
    loza.loza_ssa_calibration_alpha_grad(dout, o_full, o_sparse, again, ws)
    torch.cuda.synchronize()
    assert torch.equal(again, dalpha)                      # deterministic


def test_alpha_gradient_after_the_calibration_forward(gpu_device):
    """The tensors the calibration forward wrote, fed to the gradient; held against the oracle's two
    attentions (unrounded), so the bound is the bf16 rounding of O and O' summed over the elements."""
    B, S, Hq, s, l, b, alpha = 1, 300, 64, 1, 2, 32, 0.3
    q = _rand((B, S, Hq, 576), 51, torch.bfloat16, gpu_device)
    k = _rand((B, S, 1, 576), 52, torch.bfloat16, gpu_device)
    scale = 192 ** -0.5
    out, o_full, o_sparse, _, _ = _run(q, k, k, s, l, b, alpha, scale, 512)
    dout = _rand(out.shape, 53, torch.bfloat16, gpu_device)
    dalpha = torch.empty(1, dtype=torch.float32, device=gpu_device)
    ws = torch.empty(loza.loza_ssa_calibration_alpha_grad_workspace_bytes(out.numel()), dtype=torch.uint8, device=gpu_device)
    loza.loza_ssa_calibration_alpha_grad(dout, o_full, o_sparse, dalpha, ws)
    torch.cuda.synchronize()
    rb, rh, ri = H.all_rows(B, Hq, S)
    qr = q[torch.as_tensor(rb, device=gpu_device), torch.as_tensor(ri, device=gpu_device), torch.as_tensor(rh, device=gpu_device)].contiguous().cpu()
    _, r_full, r_sparse, _, _ = oracle.calibration_rows(qr, k.cpu(), ("alias", 512), rb, rh, ri, Hq=Hq, sink_blocks=s, local_blocks=l,
                                                        block=b, alpha=alpha, scale=scale)
    d_rows = dout[torch.as_tensor(rb, device=gpu_device), torch.as_tensor(ri, device=gpu_device), torch.as_tensor(rh, device=gpu_device)].double().cpu().numpy()
    ref = oracle.calibration_alpha_grad(d_rows, r_full, r_sparse)
    # each of the n terms carries the rounding of O and of O' (and the kernels' own 1e-2-bounded error): a random sum
    bound = 6.0 * np.sqrt(d_rows.size) * 2.0 ** -8 * float(np.abs(d_rows).mean()) * float(np.abs(r_full).mean() + np.abs(r_sparse).mean())
    print(f"[parity] alpha gradient after the forward: got {float(dalpha.item()):.6g} ref {ref:.6g} bound {bound:.3g}", flush=True)
    assert abs(float(dalpha.item()) - ref) <= bound
