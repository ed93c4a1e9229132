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
    (1, 1, 64, 0, 1, None),         # a single position
    (3, 5, 64, 1, 1, None),         # window of one token: every query sees itself and the sink token
    (1, 70, 128, 4, 20, None),      # 128 heads on one latent: a position is four row tiles
    (1, 90, 96, 2, 30, None),       # 96 heads: a position is three row tiles
    (1, 300, 64, 2, 2, 64),         # two sink blocks = two key tiles with sink keys, each cut in chunks
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
    (1, 200, 32, 1, False, 8, 40, None),     # 32 heads per group: one row tile per position
    (2, 129, 2, 2, True, 0, 128, None),      # window as long as the sequence minus one
    (1, 64, 4, 2, False, 1, 1, 64),          # one block holds everything
])
def test_d128_backward(gpu_device, B, S, Hq, Hkv, alias, ns, win, block):
    q, k, v, dout = _case(gpu_device, B, S, Hq, Hkv, 128, 128, alias)
    scale = 128 ** -0.5
    out, lse = H.oracle_forward_all(q, k, v, ns, win, scale, 128, block)
    got = H.run_backward(q, k, v, out, lse, dout, ns, win, scale, block)
    H.compare_backward(q, k, v, out, lse, dout, got, ns, win, scale,
                       f"d128 bwd B{B} S{S} Hq{Hq} Hkv{Hkv} alias{alias} ns{ns} W{win} b{block}", block)


def test_mla_backward_dense_gradient_over_several_sink_chunks(gpu_device):
    """Every row contributes (dense dO) at a length where a key tile with sink keys is seen by several
    chunks of rows (their fp32 partial tiles are summed by the reduce kernel) and the key tiles of a
    window are many: S = 2048, 64 heads on one latent, 128 sink tokens, window 512."""
    import paper_2512_23966_amd as loza
    B, S, Hq, ns, win = 1, 2048, 64, 128, 512
    q, k, v, dout = _case(gpu_device, B, S, Hq, 1, 576, 512, alias=True, seed=50)
    scale = 192 ** -0.5
    # the schedule really has more than one chunk per sink tile: the workspace holds their partial tiles
    stat_only = B * 1 * ((S * Hq + 31) // 32 * 32) * 8
    assert loza.loza_ssa_backward_workspace_bytes(B, Hq, 1, S, 576, 512, ns, win, True) > stat_only + 2 * 64 * 576 * 4
    out, lse = H.oracle_forward_all(q, k, v, ns, win, scale, 512)
    got = H.run_backward(q, k, v, out, lse, dout, ns, win, scale)
    H.compare_backward(q, k, v, out, lse, dout, got, ns, win, scale, f"mla bwd dense S{S} ns{ns} W{win}")


def test_mla_backward_two_latent_heads(gpu_device):
    B, S, Hq, Hkv, ns, win = 2, 70, 128, 2, 4, 20
    q, k, v, dout = _case(gpu_device, B, S, Hq, Hkv, 576, 512, alias=True, seed=30)
    scale = 192 ** -0.5
    out, lse = H.oracle_forward_all(q, k, v, ns, win, scale, 512)
    got = H.run_backward(q, k, v, out, lse, dout, ns, win, scale)
    H.compare_backward(q, k, v, out, lse, dout, got, ns, win, scale, "mla bwd two latent heads")


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


def test_backward_at_the_128k_prefill_shape(gpu_device):
    """S = 131072, 64 heads on one latent, sink 128 + window 8192: the launch the benchmark times.
    The incoming gradient is zero outside a sample of rows, so the oracle can follow every one of
    the 131072 dK rows (each is a sum over the sampled rows that see that key) and the sampled dQ
    rows; every other dQ row must come out exactly zero. The device does the full work either way."""
    cfg = W.CFG3
    q, k, v = W.make_prefill_inputs(cfg, gpu_device)
    assert v is k
    rb, rh, ri = W.sample_rows(cfg, n_random=24, n_heads=3, edge=4)
    n = len(rb)
    idx = (torch.as_tensor(rb, device=gpu_device), torch.as_tensor(ri, device=gpu_device), torch.as_tensor(rh, device=gpu_device))
    q_rows = q[idx].contiguous().cpu()
    g = torch.Generator().manual_seed(77)
    dout_rows = torch.randn((n, cfg.d_v), generator=g, dtype=torch.float32).to(torch.bfloat16)
    # what a forward pass would have stored for those rows, from the oracle's forward
    o_rows, l_rows = oracle.ssa_rows(q_rows, k.cpu(), ("alias", cfg.d_v), rb, rh, ri, Hq=cfg.Hq, n_sink=cfg.n_sink,
                                     window=cfg.window, scale=cfg.scale)
    out_rows = torch.as_tensor(o_rows).to(torch.bfloat16)
    lse_rows = torch.as_tensor(l_rows).to(torch.float32)
    dout = torch.zeros(cfg.B, cfg.S, cfg.Hq, cfg.d_v, dtype=torch.bfloat16, device=gpu_device)
    out = torch.zeros_like(dout)
    lse = torch.full((cfg.B, cfg.Hq, cfg.S), 1.0e4, dtype=torch.float32, device=gpu_device)  # weights of the other rows: 0
    dout[idx] = dout_rows.to(gpu_device)
    out[idx] = out_rows.to(gpu_device)
    lse[idx[0], idx[2], idx[1]] = lse_rows.to(gpu_device)
    dq, dk, _ = H.run_backward(q, k, v, out, lse, dout, cfg.n_sink, cfg.window, cfg.scale)
    rq, rk, rv = oracle.ssa_backward_rows(q_rows, k.cpu(), ("alias", cfg.d_v), dout_rows, rb, rh, ri, Hq=cfg.Hq,
                                          n_sink=cfg.n_sink, window=cfg.window, scale=cfg.scale,
                                          out_rows=out_rows, lse_rows=lse_rows)
    rk[..., :cfg.d_v] += rv
    got_q = dq[idx].double().cpu().numpy()
    got_k = dk.double().cpu().numpy()
    assert np.isfinite(got_q).all() and np.isfinite(got_k).all()
    for name, gg, r in (("dq (sampled rows)", got_q, rq), ("dk (all keys)", got_k, rk)):
        err = np.abs(gg - r)
        over = float((err - H.grad_tolerance(r)).max())
        print(f"[parity] cfg3 backward, {n} rows with a gradient: {name} max|err|={err.max():.3e} "
              f"max|ref|={np.abs(r).max():.3e}", flush=True)
        assert over <= 0.0, f"{name}: error exceeds its bound by {over}"
    # rows without an incoming gradient: exactly zero, and all of them written. (A sampled row whose
    # true gradient is zero -- position 0 sees one key, so dP = D -- may come out as exact zeros too.)
    nonzero = (dq != 0).any(dim=-1)
    sampled = torch.zeros_like(nonzero)
    sampled[idx] = True
    must = torch.zeros_like(nonzero)
    has_grad = torch.as_tensor((rq != 0).any(axis=-1), device=gpu_device)
    must[idx[0][has_grad], idx[1][has_grad], idx[2][has_grad]] = True
    assert not (nonzero & ~sampled).any(), "a row without an incoming gradient has a non-zero dq"
    assert (nonzero | ~must).all(), "a row with a gradient came out as zeros"
    assert torch.isfinite(dq.float().sum())
