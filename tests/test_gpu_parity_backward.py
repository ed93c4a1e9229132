"""GPU parity of the SSA backward (dq, dk, dv over live pairs only) against the oracle's gradient.
Both take the same stored `out` (bf16) and `lse` (fp32) as a training step does; these come from the
oracle's forward, never from the HIP forward. One test chains HIP forward and HIP backward instead
and holds the result against the oracle's gradient from the definition alone."""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_23966_amd import workloads as W
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _rand(shape, seed, device, scale=1.0):
    g = torch.Generator(device=device).manual_seed(seed)
    return (torch.randn(shape, generator=g, device=device, dtype=torch.float32) * scale).to(torch.bfloat16)


def _case(device, B, S, Hq, Hkv, d_qk, d_v, alias, seed=0):
    q = _rand((B, S, Hq, d_qk), seed + 1, device)
    k = _rand((B, S, Hkv, d_qk), seed + 2, device)
    v = k if alias else _rand((B, S, Hkv, d_v), seed + 3, device)
    dout = _rand((B, S, Hq, d_v), seed + 4, device)
    return q, k, v, dout


@pytest.mark.parametrize("B,S,Hq,ns,win,block", [
    (1, 160, 64, 16, 40, None),     # the absorbed-MLA head layout: 64 heads on one latent
    (1, 200, 64, 8, 8, None),       # sink key tile seen by many row chunks (partial sums + reduce)
    (2, 97, 32, 0, 33, None),       # no sink, ragged last tiles, two sequences
    (1, 130, 64, 1, 2, 32),         # block-granular
    (1, 150, 64, 7, None, None),    # window = infinity: causal attention
    (1, 33, 64, 40, 5, None),       # more sink tokens than keys
])
def test_mla_backward(gpu_device, B, S, Hq, ns, win, block):
    q, k, v, dout = _case(gpu_device, B, S, Hq, 1, 576, 512, alias=True)
    scale = 192 ** -0.5
    out, lse = H.oracle_forward_all(q, k, v, ns, win, scale, 512, block)
    got = H.run_backward(q, k, v, out, lse, dout, ns, win, scale, block)
    H.compare_backward(q, k, v, out, lse, dout, got, ns, win, scale, f"mla bwd B{B} S{S} Hq{Hq} ns{ns} W{win} b{block}", block)


@pytest.mark.parametrize("B,S,Hq,Hkv,alias,ns,win,block", [
    (1, 300, 4, 4, False, 16, 50, None),     # MHA: one head per group
    (2, 257, 8, 2, False, 4, 31, None),      # grouped heads (4 per group), ragged
    (1, 400, 2, 1, True, 32, 64, None),      # aliased values of equal width
    (1, 260, 16, 1, False, 1, 3, 20),        # block-granular, 16 heads per group
    (1, 2500, 1, 1, False, 64, 128, None),   # long enough for several row chunks of the sink tile at G = 1
])
def test_d128_backward(gpu_device, B, S, Hq, Hkv, alias, ns, win, block):
    q, k, v, dout = _case(gpu_device, B, S, Hq, Hkv, 128, 128, alias)
    scale = 128 ** -0.5
    out, lse = H.oracle_forward_all(q, k, v, ns, win, scale, 128, block)
    got = H.run_backward(q, k, v, out, lse, dout, ns, win, scale, block)
    H.compare_backward(q, k, v, out, lse, dout, got, ns, win, scale,
                       f"d128 bwd B{B} S{S} Hq{Hq} Hkv{Hkv} alias{alias} ns{ns} W{win} b{block}", block)


def test_backward_after_the_hip_forward(gpu_device):
    """The chain a training step runs: HIP forward, then HIP backward fed with its out and lse."""
    q, k, v, dout = _case(gpu_device, 1, 192, 64, 1, 576, 512, alias=True, seed=10)
    ns, win, scale = 16, 64, 192 ** -0.5
    out, lse = H.run_prefill(q, k, v, ns, win, scale, d_v=512)
    dq, dk, _ = H.run_backward(q, k, v, out, lse, dout, ns, win, scale)
    # against the gradient from the definition (the oracle recomputes its own forward in fp64): on top
    # of the kernel's own rounding this sees the bf16 rounding of the stored `out` inside
    # D_i = dout_i . out_i, an error of about 2^-9 |dout_i| |out_i| that enters every dS of the row
    rq, rk, rv = oracle.ssa_backward(q.cpu(), k.cpu(), ("alias", 512), dout.cpu(), n_sink=ns, window=win, scale=scale)
    rk[..., :512] += rv
    for name, g, r in (("dq", dq, rq), ("dk", dk, rk)):
        err = np.abs(g.double().cpu().numpy() - r)
        rel = np.sqrt((err ** 2).mean()) / np.sqrt((r ** 2).mean())
        print(f"[parity] mla fwd+bwd chain: {name} rms error / rms gradient = {rel:.2e}, max|err|={err.max():.3e}, "
              f"max|gradient|={np.abs(r).max():.3e}", flush=True)
        assert rel < 2.0 ** -7 and err.max() < 2.0 ** -6 * np.abs(r).max()


def test_backward_is_deterministic(gpu_device):
    q, k, v, dout = _case(gpu_device, 1, 200, 64, 1, 576, 512, alias=True, seed=20)
    ns, win, scale = 8, 8, 192 ** -0.5
    out, lse = H.run_prefill(q, k, v, ns, win, scale, d_v=512)
    a = H.run_backward(q, k, v, out, lse, dout, ns, win, scale)
    b = H.run_backward(q, k, v, out, lse, dout, ns, win, scale)
    assert torch.equal(a[0].view(torch.int16), b[0].view(torch.int16))
    assert torch.equal(a[1].view(torch.int16), b[1].view(torch.int16))


def test_unsupported_group_size_is_refused(gpu_device):
    import paper_2512_23966_amd as loza
    q, k, v, dout = _case(gpu_device, 1, 64, 3, 1, 128, 128, alias=False)
    out = torch.zeros_like(dout)
    lse = torch.zeros(1, 3, 64, dtype=torch.float32, device=gpu_device)
    with pytest.raises(loza.LozaError) as e:
        H.run_backward(q, k, v, out, lse, dout, 4, 16, 0.1)
    assert "UNSUPPORTED" in str(e.value)
