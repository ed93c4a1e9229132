"""GPU parity of the fp32 SSA backward against the oracle's gradient (both take the same stored out
and lse, which come from the oracle's forward)."""
import pytest
import torch

from tests import helpers as H

pytestmark = pytest.mark.gpu


def _rand(shape, seed, device):
    g = torch.Generator(device=device).manual_seed(seed)
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32)


@pytest.mark.parametrize("B,S,Hq,Hkv,d_qk,d_v,alias,ns,win,block", [
    (1, 1024, 1, 1, 64, 64, False, 64, 256, None),   # the tiny fp32 configuration
    (2, 150, 4, 2, 64, 32, False, 3, 17, None),      # grouped heads, d_v < d_qk, ragged
    (1, 200, 2, 1, 96, 64, True, 8, 40, None),       # values are a prefix of the key rows
    (1, 130, 3, 3, 40, 24, False, 0, 1, None),       # no sink, window of one, odd widths
    (1, 90, 2, 2, 256, 256, False, 100, 5, None),    # widest rows; more sink tokens than keys
    (1, 300, 2, 1, 32, 32, False, 1, 2, 32),         # block-granular
    (1, 77, 5, 1, 16, 16, True, 2, None, None),      # window = infinity, five heads on one kv head
    (3, 1, 2, 2, 8, 8, False, 0, 1, None),           # a single position
])
def test_backward_f32(gpu_device, B, S, Hq, Hkv, d_qk, d_v, alias, ns, win, block):
    q = _rand((B, S, Hq, d_qk), 1, gpu_device)
    k = _rand((B, S, Hkv, d_qk), 2, gpu_device)
    v = k if alias else _rand((B, S, Hkv, d_v), 3, gpu_device)
    dout = _rand((B, S, Hq, d_v), 4, gpu_device)
    scale = d_qk ** -0.5
    out, lse = H.oracle_forward_all_f32(q, k, v, ns, win, scale, d_v, block)
    got = H.run_backward_f32(q, k, v, out, lse, dout, ns, win, scale, block)
    H.compare_backward_f32(q, k, v, out, lse, dout, got, ns, win, scale,
                           f"f32 bwd B{B} S{S} Hq{Hq}/{Hkv} d{d_qk}/{d_v} alias{alias} ns{ns} W{win} b{block}", block)


def test_backward_f32_after_the_hip_forward(gpu_device):
    """HIP fp32 forward, then HIP fp32 backward on what it stored, against the oracle's gradient
    from the definition alone."""
    B, S, Hq, Hkv, d, ns, win = 1, 256, 2, 1, 64, 16, 50
    q, k, v, dout = (_rand(s, i, gpu_device) for i, s in enumerate(
        [(B, S, Hq, d), (B, S, Hkv, d), (B, S, Hkv, d), (B, S, Hq, d)], start=10))
    scale = d ** -0.5
    out, lse = H.run_prefill(q, k, v, ns, win, scale)
    got = H.run_backward_f32(q, k, v, out, lse, dout, ns, win, scale)
    import numpy as np
    import oracle
    rq, rk, rv = oracle.ssa_backward(q.cpu(), k.cpu(), v.cpu(), dout.cpu(), n_sink=ns, window=win, scale=scale)
    for name, g, r in (("dq", got[0], rq), ("dk", got[1], rk), ("dv", got[2], rv)):
        err = np.abs(g.double().cpu().numpy() - r)
        assert float((err - 2.0 * H.grad_tolerance_f32(r)).max()) <= 0.0, f"{name}: max error {err.max()}"
