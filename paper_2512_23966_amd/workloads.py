"""Synthetic workloads: the five benchmark configurations, seeded input generators, row samples.

This module holds no arithmetic of the attention method. It only says what the inputs look like
(shapes, value distribution, seeds) and which output rows a sampled comparison looks at; both the
HIP path and the CPU oracle are fed from the tensors made here, so they see the same bits.

The paper measures on no public dataset for this path (its efficiency figure times kernels and a
serving engine); these configurations reuse its context lengths (32K / 128K / 256K trained, 1M by
extrapolation — Training section) with iid N(0,1) values, and stand in for its workloads.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional

import numpy as np
import torch

INF = None  # window=None means "infinite": full causal attention


@dataclass(frozen=True)
class PrefillConfig:
    name: str
    dtype: torch.dtype
    B: int
    Hq: int
    Hkv: int
    S: int
    d_qk: int
    d_v: int
    alias_v: bool          # values are the first d_v columns of the keys (absorbed MLA latent)
    n_sink: int
    window: Optional[int]
    scale: float
    seed: int


@dataclass(frozen=True)
class DecodeConfig:
    name: str
    B: int
    Hq: int
    Hkv: int
    S_max: int
    len_lo: int
    len_hi: int
    d_qk: int
    d_v: int
    alias_v: bool
    n_sink: int
    window: Optional[int]
    scale: float
    seed: int


CFG1 = PrefillConfig("cfg1_tiny_f32_prefill", torch.float32, 1, 1, 1, 1024, 64, 64, False, 64, 256, 64 ** -0.5, 0)
CFG2 = PrefillConfig("cfg2_mha_bf16_prefill_32k", torch.bfloat16, 1, 32, 32, 32768, 128, 128, False, 128, 4096, 128 ** -0.5, 1)
CFG3 = PrefillConfig("cfg3_mla_bf16_prefill_128k", torch.bfloat16, 1, 64, 1, 131072, 576, 512, True, 128, 8192, 192 ** -0.5, 2)
CFG4 = DecodeConfig("cfg4_mla_bf16_decode_b64", 64, 64, 1, 262144, 65536, 262144, 576, 512, True, 128, 8192, 192 ** -0.5, 3)
CFG5 = PrefillConfig("cfg5_mla_bf16_prefill_1m", torch.bfloat16, 1, 64, 1, 1048576, 576, 512, True, 128, 8192, 192 ** -0.5, 4)
# the full-attention comparator of the 1M configuration: window = infinity on its first 131072 tokens
CFG5_FULL_128K = replace(CFG3, name="cfg5cmp_mla_bf16_full_128k", window=INF, seed=4)


def full_attention(cfg):
    """The same workload with window = infinity (the full-attention comparator)."""
    return replace(cfg, name=cfg.name + "_full", window=INF)


def _fill_normal(t: torch.Tensor, gen: torch.Generator, chunk: int = 1 << 26) -> None:
    """t <- iid N(0,1) drawn in fp32 and rounded to t.dtype (round to nearest even), chunk by chunk."""
    flat = t.view(-1)
    n = flat.numel()
    for a in range(0, n, chunk):
        b = min(n, a + chunk)
        flat[a:b].copy_(torch.randn(b - a, generator=gen, device=t.device, dtype=torch.float32))


def make_prefill_inputs(cfg: PrefillConfig, device):
    """(q, k, v): q [B,S,Hq,d_qk], k [B,S,Hkv,d_qk], v [B,S,Hkv,d_v] — ``v is k`` when alias_v."""
    device = torch.device(device)
    gen = torch.Generator(device=device).manual_seed(cfg.seed)
    q = torch.empty(cfg.B, cfg.S, cfg.Hq, cfg.d_qk, dtype=cfg.dtype, device=device)
    k = torch.empty(cfg.B, cfg.S, cfg.Hkv, cfg.d_qk, dtype=cfg.dtype, device=device)
    _fill_normal(q, gen)
    _fill_normal(k, gen)
    if cfg.alias_v:
        v = k
    else:
        v = torch.empty(cfg.B, cfg.S, cfg.Hkv, cfg.d_v, dtype=cfg.dtype, device=device)
        _fill_normal(v, gen)
    return q, k, v


def make_decode_inputs(cfg: DecodeConfig, device, poison_tail: bool = False):
    """(q, kcache, vcache, seqlens): one new query token per sequence against its cache.

    seqlens are seeded integers uniform in [len_lo, len_hi]; cache rows at or beyond a sequence's
    length are filled too (with N(0,1), or with NaN when ``poison_tail`` — they must never be read).
    """
    device = torch.device(device)
    gen = torch.Generator(device=device).manual_seed(cfg.seed)
    rng = np.random.default_rng(cfg.seed)
    seqlens_np = rng.integers(cfg.len_lo, cfg.len_hi + 1, size=cfg.B).astype(np.int32)
    q = torch.empty(cfg.B, cfg.Hq, cfg.d_qk, dtype=torch.bfloat16, device=device)
    kc = torch.empty(cfg.B, cfg.S_max, cfg.Hkv, cfg.d_qk, dtype=torch.bfloat16, device=device)
    _fill_normal(q, gen)
    _fill_normal(kc, gen)
    if cfg.alias_v:
        vc = kc
    else:
        vc = torch.empty(cfg.B, cfg.S_max, cfg.Hkv, cfg.d_v, dtype=torch.bfloat16, device=device)
        _fill_normal(vc, gen)
    if poison_tail:
        for b, L in enumerate(seqlens_np.tolist()):
            kc[b, L:] = float("nan")
            if vc is not kc:
                vc[b, L:] = float("nan")
    seqlens = torch.from_numpy(seqlens_np).to(device)
    return q, kc, vc, seqlens


def sample_rows(cfg: PrefillConfig, n_random: int = 256, n_heads: int = 4, edge: int = 64, seed: int = 12345):
    """Deterministic sample of (b, h, i) output rows for comparisons at sizes the oracle cannot sweep.

    Positions: the first and last ``edge`` rows, every position where the live set changes shape
    (around n_sink, window, n_sink + window), positions around workgroup-tile boundaries, and
    ``n_random`` seeded random positions. Heads: ``n_heads`` of them, always head 0 and Hq - 1.
    """
    S, ns = cfg.S, cfg.n_sink
    W = S if cfg.window is None else min(cfg.window, S)
    T = ns + W
    pos = set(range(0, min(edge, S))) | set(range(max(0, S - edge), S))
    for c in (ns, W, T, 128, 256, 4096, S // 2, S // 2 + 64):
        for d in (-2, -1, 0, 1, 2):
            if 0 <= c + d < S:
                pos.add(c + d)
    rng = np.random.default_rng(seed)
    if n_random > 0:
        pos |= set(int(x) for x in rng.integers(0, S, size=n_random))
    pos = sorted(pos)
    heads = sorted({0, cfg.Hq - 1} | set(int(x) for x in rng.integers(0, cfg.Hq, size=max(0, n_heads - 2))))
    b, h, i = np.meshgrid(np.arange(cfg.B), np.asarray(heads), np.asarray(pos), indexing="ij")
    return b.ravel().astype(np.int64), h.ravel().astype(np.int64), i.ravel().astype(np.int64)
