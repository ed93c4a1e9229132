"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

The oracle cannot sweep these sizes, and output rows are independent of each other, so each
configuration is compared on a deterministic row sample (paper_2512_23966_amd.workloads.sample_rows:
first/last rows, every position where the live set changes shape, workgroup-tile boundaries, seeded
random rows) — every sampled row is computed by the oracle one by one from the very bits on the GPU.
"""
import numpy as np
import pytest
import torch

from paper_2512_23966_amd import workloads as W
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _prefill_case(cfg, dev, n_random, n_heads):
    print(f"\n[case] {cfg.name}: generating inputs", flush=True)
    q, k, v = W.make_prefill_inputs(cfg, dev)
    out, lse = H.run_prefill(q, k, v, cfg.n_sink, cfg.window, cfg.scale, d_v=cfg.d_v)
    rb, rh, ri = W.sample_rows(cfg, n_random=n_random, n_heads=n_heads)
    print(f"[case] {cfg.name}: oracle on {len(rb)} sampled rows", flush=True)
    res = H.compare_prefill(q, k, v, out, lse, rb, rh, ri, cfg.n_sink, cfg.window, cfg.scale, cfg.name)
    del q, k, v, out, lse
    torch.cuda.empty_cache()
    return res


def test_cfg2_mha_bf16_prefill_32k(gpu_device):
    _prefill_case(W.CFG2, gpu_device, n_random=256, n_heads=4)


def test_cfg3_mla_bf16_prefill_128k(gpu_device):
    _prefill_case(W.CFG3, gpu_device, n_random=256, n_heads=4)


def test_cfg3_full_attention_comparator_128k(gpu_device):
    _prefill_case(W.CFG5_FULL_128K, gpu_device, n_random=48, n_heads=2)


def test_cfg5_mla_bf16_prefill_1m(gpu_device):
    free, _ = torch.cuda.mem_get_info()
    if free < 160 * 2 ** 30:
        pytest.skip("the 1M-token configuration needs 150 GB of free HBM")
    _prefill_case(W.CFG5, gpu_device, n_random=192, n_heads=3)


def test_cfg4_mla_bf16_decode_b64(gpu_device):
    cfg = W.CFG4
    print(f"\n[case] {cfg.name}: generating inputs", flush=True)
    q, kc, vc, seqlens = W.make_decode_inputs(cfg, gpu_device, poison_tail=True)
    out, lse = H.run_decode(q, kc, vc, seqlens, cfg.n_sink, cfg.window, cfg.scale, d_v=cfg.d_v)
    # every sequence, 6 heads each (always the first and the last)
    heads = np.asarray([0, 1, 17, 31, 32, 63], dtype=np.int64)
    rb = np.repeat(np.arange(cfg.B, dtype=np.int64), len(heads))
    rh = np.tile(heads, cfg.B)
    print(f"[case] {cfg.name}: oracle on {len(rb)} sampled rows", flush=True)
    H.compare_decode(q, kc, vc, seqlens, out, lse, rb, rh, cfg.n_sink, cfg.window, cfg.scale, cfg.name)
    assert torch.isfinite(out.float()).all() and torch.isfinite(lse).all()


def test_cfg4_decode_full_attention_comparator(gpu_device):
    cfg = W.CFG4
    q, kc, vc, seqlens = W.make_decode_inputs(cfg, gpu_device, poison_tail=True)
    out, lse = H.run_decode(q, kc, vc, seqlens, cfg.n_sink, None, cfg.scale, d_v=cfg.d_v)
    rb = np.asarray([0, 0, 21, 63, 63], dtype=np.int64)
    rh = np.asarray([0, 63, 30, 5, 63], dtype=np.int64)
    H.compare_decode(q, kc, vc, seqlens, out, lse, rb, rh, cfg.n_sink, None, cfg.scale, cfg.name + "_full")
