"""Shared plumbing of the GPU parity tests: call the HIP path through the C ABI binding, call the
fp64 oracle on the same bits, compare element by element."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2512_23966_amd as loza

# Tolerances (max abs error against the fp64 oracle). bf16 paths: 1e-2 on the output; fp32 path: 1e-5
# on output and log-sum-exp. The log-sum-exp of the bf16 paths is fp32 arithmetic throughout (scores
# by fp32-accumulating matrix cores, fp32 exponentials and sums): measured error 1e-6 .. 3e-6, bound
# 2e-5. That is tight enough to count keys: one key too many or too few among n_sink + window =
# 8320 equally weighted ones moves it by ln(8321 / 8320) = 1.2e-4.
TOL = {torch.bfloat16: (1e-2, 2e-5), torch.float32: (1e-5, 1e-5)}
# Results of magnitude 2 and more come from the two-term-weights pass (prefill, extend) or from the
# fp32 direct path (decode): what their arithmetic may add to the rounding of the result to bf16 is
# relative to the result: weights good to 2^-17, fp32 sums over up to 2^18 terms.
BF16_ARITH_REL = 2.0 ** -12


def out_tolerance(ref: np.ndarray, dtype) -> np.ndarray:
    """Element-wise bound on |out - ref|: the flat bound of the task (1e-2 for bf16) wherever the
    rounding of the result to bf16 leaves room for it, i.e. for |ref| < 4 (half an ulp is 2^-7 =
    7.8e-3 for |ref| in [2, 4)). From 4 on half an ulp alone is 2^-6 = 1.6e-2, which rows with two or
    three live keys of N(0,1) values do reach: there the bound is that half ulp plus 2^-12 |ref|."""
    flat = TOL[dtype][0]
    if dtype != torch.bfloat16:
        return np.full(ref.shape, flat)
    mag = np.maximum(np.abs(ref), 1e-30)
    half_ulp = np.exp2(np.floor(np.log2(mag)) - 8.0)
    return np.maximum(flat, half_ulp + BF16_ARITH_REL * mag)


def live_count_tokens(i, n_sink, window):
    """|live(i)| of the token-granular pattern in closed form: min(i + 1, n_sink + window).
    (tests/test_oracle_pins.py holds it against the oracle's explicit mask.)"""
    return np.minimum(i + 1, n_sink + window)


def live_count_blocks(i, sink_blocks, local_blocks, block):
    """|live(i)| of the block-granular pattern in closed form: the sink tokens that lie before the
    window, plus the window's keys up to the query (the window starts local_blocks - 1 blocks before
    the query's block). (tests/test_oracle_pins_blocks.py holds it against the oracle's explicit mask.)"""
    wb = np.maximum(0, i // block - local_blocks + 1) * block
    se = np.minimum(i + 1, sink_blocks * block)
    return np.minimum(se, wb) + (i + 1 - wb)


def run_prefill(q, k, v, n_sink, window, scale, d_v=None, block=None):
    """``block=None``: token-granular (n_sink, window in tokens); ``block=b``: block-granular, n_sink and
    window then count blocks of b tokens."""
    B, S, Hq, _ = q.shape
    d_v = d_v if d_v is not None else v.shape[3]
    out = torch.empty(B, S, Hq, d_v, dtype=q.dtype, device=q.device)
    lse = torch.empty(B, Hq, S, dtype=torch.float32, device=q.device)
    if block is None:
        fn = loza.loza_ssa_prefill if q.dtype == torch.bfloat16 else loza.loza_ssa_prefill_f32
        fn(q, k, v, out, lse, n_sink, window, scale)
    else:
        fn = loza.loza_ssa_prefill_blocks if q.dtype == torch.bfloat16 else loza.loza_ssa_prefill_blocks_f32
        fn(q, k, v, out, lse, n_sink, window, block, scale)
    torch.cuda.synchronize()
    return out, lse


def run_decode(q, kc, vc, seqlens, n_sink, window, scale, d_v=None, block=None):
    B, Hq, _ = q.shape
    _, S_max, Hkv, _ = kc.shape
    d_v = d_v if d_v is not None else vc.shape[3]
    out = torch.empty(B, Hq, d_v, dtype=torch.bfloat16, device=q.device)
    lse = torch.empty(B, Hq, dtype=torch.float32, device=q.device)
    if block is None:
        nbytes = loza.loza_ssa_decode_workspace_bytes(B, Hq, Hkv, S_max, d_v, n_sink, window)
        ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=q.device)
        loza.loza_ssa_decode(q, kc, vc, seqlens, out, lse, n_sink, window, scale, ws)
    else:
        w_tokens = None if window is None else window * block
        nbytes = loza.loza_ssa_decode_workspace_bytes(B, Hq, Hkv, S_max, d_v, n_sink * block, w_tokens)
        ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=q.device)
        loza.loza_ssa_decode_blocks(q, kc, vc, seqlens, out, lse, n_sink, window, block, scale, ws)
    torch.cuda.synchronize()
    return out, lse


def run_decode_f32(q, kc, vc, seqlens, n_sink, window, scale, d_v=None, block=None):
    B, Hq, _ = q.shape
    d_v = d_v if d_v is not None else vc.shape[3]
    out = torch.full((B, Hq, d_v), float("nan"), dtype=torch.float32, device=q.device)
    lse = torch.full((B, Hq), float("nan"), dtype=torch.float32, device=q.device)
    if block is None:
        loza.loza_ssa_decode_f32(q, kc, vc, seqlens, out, lse, n_sink, window, scale)
    else:
        loza.loza_ssa_decode_blocks_f32(q, kc, vc, seqlens, out, lse, n_sink, window, block, scale)
    torch.cuda.synchronize()
    return out, lse


def oracle_prefill_rows(q, k, v, rb, rh, ri, n_sink, window, scale, d_v, block=None):
    """Oracle on the listed (b, h, i) rows, fed with the very bits the GPU tensors hold."""
    idx = (torch.as_tensor(rb, device=q.device), torch.as_tensor(ri, device=q.device), torch.as_tensor(rh, device=q.device))
    q_rows = q[idx].contiguous().cpu()
    varg = ("alias", d_v) if v is k else v.cpu()
    w = oracle.INT64_MAX if window is None else window
    return oracle.ssa_rows(q_rows, k.cpu(), varg, rb, rh, ri, Hq=q.shape[2], n_sink=n_sink, window=w, scale=scale,
                           block=block)


def all_rows(B, Hq, S):
    b, h, i = np.meshgrid(np.arange(B), np.arange(Hq), np.arange(S), indexing="ij")
    return b.ravel().astype(np.int64), h.ravel().astype(np.int64), i.ravel().astype(np.int64)


def compare_prefill(q, k, v, out, lse, rb, rh, ri, n_sink, window, scale, label="", block=None):
    d_v = out.shape[3]
    ref_out, ref_lse = oracle_prefill_rows(q, k, v, rb, rh, ri, n_sink, window, scale, d_v, block)
    dev = q.device
    idx = (torch.as_tensor(rb, device=dev), torch.as_tensor(ri, device=dev), torch.as_tensor(rh, device=dev))
    got_out = out[idx].double().cpu().numpy()
    got_lse = lse[torch.as_tensor(rb, device=dev), torch.as_tensor(rh, device=dev), torch.as_tensor(ri, device=dev)].double().cpu().numpy()
    assert np.isfinite(got_out).all(), f"{label}: non-finite output"
    return _judge(got_out, ref_out, got_lse, ref_lse, q.dtype, len(rb), label)


def _judge(got_out, ref_out, got_lse, ref_lse, dtype, n_rows, label):
    err = np.abs(got_out - ref_out)
    e_out = float(err.max())
    e_lse = float(np.abs(got_lse - ref_lse).max())
    tol_out, tol_lse = TOL[dtype]
    big = int((np.abs(ref_out) >= 4.0).sum())
    print(f"[parity] {label}: rows={n_rows} max|out err|={e_out:.3e} (tol {tol_out}; {big} results of magnitude >= 4 "
          f"take their bf16 half ulp) max|lse err|={e_lse:.3e} (tol {tol_lse})", flush=True)
    worst = float((err - out_tolerance(ref_out, dtype)).max())
    assert worst <= 0.0, f"{label}: out error exceeds its bound by {worst} (max error {e_out})"
    assert e_lse <= tol_lse, f"{label}: lse error {e_lse} > {tol_lse}"
    return e_out, e_lse


def oracle_decode(q, kc, vc, seqlens, rb, rh, n_sink, window, scale, d_v, block=None):
    """Oracle for decode rows (b, h): the query sits at position seqlens[b] - 1 of its cache."""
    L = seqlens.cpu().numpy().astype(np.int64)
    ri = L[rb] - 1
    q_rows = q[torch.as_tensor(rb, device=q.device), torch.as_tensor(rh, device=q.device)].contiguous().cpu()
    # NaN-poisoned rows beyond the length must not reach the oracle's arithmetic either: it never
    # touches a dead key, so the cache is passed as is
    varg = ("alias", d_v) if vc is kc else vc.cpu()
    w = oracle.INT64_MAX if window is None else window
    return oracle.ssa_rows(q_rows, kc.cpu(), varg, rb, rh, ri, Hq=q.shape[1], n_sink=n_sink, window=w, scale=scale,
                           block=block)


def compare_decode(q, kc, vc, seqlens, out, lse, rb, rh, n_sink, window, scale, label="", block=None):
    d_v = out.shape[2]
    ref_out, ref_lse = oracle_decode(q, kc, vc, seqlens, rb, rh, n_sink, window, scale, d_v, block)
    dev = q.device
    got_out = out[torch.as_tensor(rb, device=dev), torch.as_tensor(rh, device=dev)].double().cpu().numpy()
    got_lse = lse[torch.as_tensor(rb, device=dev), torch.as_tensor(rh, device=dev)].double().cpu().numpy()
    assert np.isfinite(got_out).all(), f"{label}: non-finite output"
    return _judge(got_out, ref_out, got_lse, ref_lse, out.dtype, len(rb), label)


# ---- backward -------------------------------------------------------------------------------------

def oracle_forward_all(q, k, v, n_sink, window, scale, d_v, block=None):
    """Oracle forward of every row, shaped like the tensors the backward takes: out [B,S,Hq,d_v]
    rounded to bf16 (what a forward pass hands to the backward), lse [B,Hq,S] fp32."""
    B, S, Hq, _ = q.shape
    rb, rh, ri = all_rows(B, Hq, S)
    out, lse = oracle_prefill_rows(q, k, v, rb, rh, ri, n_sink, window, scale, d_v, block)
    out_t = torch.zeros(B, S, Hq, d_v, dtype=torch.float64)
    out_t[torch.as_tensor(rb), torch.as_tensor(ri), torch.as_tensor(rh)] = torch.as_tensor(out)
    lse_t = torch.zeros(B, Hq, S, dtype=torch.float64)
    lse_t[torch.as_tensor(rb), torch.as_tensor(rh), torch.as_tensor(ri)] = torch.as_tensor(lse)
    return out_t.to(torch.bfloat16).to(q.device), lse_t.to(torch.float32).to(q.device)


def oracle_forward_all_f32(q, k, v, n_sink, window, scale, d_v, block=None):
    """The same for fp32 tensors: out [B,S,Hq,d_v] and lse [B,Hq,S], both rounded to fp32."""
    B, S, Hq, _ = q.shape
    rb, rh, ri = all_rows(B, Hq, S)
    out, lse = oracle_prefill_rows(q, k, v, rb, rh, ri, n_sink, window, scale, d_v, block)
    out_t = torch.zeros(B, S, Hq, d_v, dtype=torch.float64)
    out_t[torch.as_tensor(rb), torch.as_tensor(ri), torch.as_tensor(rh)] = torch.as_tensor(out)
    lse_t = torch.zeros(B, Hq, S, dtype=torch.float64)
    lse_t[torch.as_tensor(rb), torch.as_tensor(rh), torch.as_tensor(ri)] = torch.as_tensor(lse)
    return out_t.to(torch.float32).to(q.device), lse_t.to(torch.float32).to(q.device)


def run_backward_f32(q, k, v, out, lse, dout, n_sink, window, scale, block=None):
    """HIP fp32 backward through the C ABI; outputs start as NaN (every element must be written)."""
    alias = v is k
    nan = float("nan")
    dq = torch.full_like(q, nan)
    dk = torch.full_like(k, nan)
    dv = None if alias else torch.full_like(v, nan)
    if block is None:
        loza.loza_ssa_backward_f32(q, k, v, out, lse, dout, dq, dk, dv, n_sink, window, scale)
    else:
        loza.loza_ssa_backward_blocks_f32(q, k, v, out, lse, dout, dq, dk, dv, n_sink, window, block, scale)
    torch.cuda.synchronize()
    return dq, dk, dv


# fp32 arithmetic throughout: the task's bound for the fp32 path, 1e-5, flat, plus 1e-5 of the element
# for gradients larger than one (fp32 holds 7 digits: an element of size 30 cannot be good to 1e-5).
# Measured: <= 6e-6. The flat part also covers the rows that vanish by cancellation: a query with one
# live key has dP = D exactly, the kernel forms both as fp32 dot products of up to 256 terms of size ~1
# in different orders (difference ~ 2^-23 * sqrt(256) * |dO||v| ~ 4e-6), and that difference times
# scale * |k| is what its dq row holds instead of zero.
def grad_tolerance_f32(ref: np.ndarray) -> np.ndarray:
    return 1e-5 + 1e-5 * np.abs(ref)


def compare_backward_f32(q, k, v, out, lse, dout, got, n_sink, window, scale, label="", block=None):
    dq, dk, dv = got
    d_v = dout.shape[3]
    alias = v is k
    w = oracle.INT64_MAX if window is None else window
    varg = ("alias", d_v) if alias else v.cpu()
    rq, rk, rv = oracle.ssa_backward(q.cpu(), k.cpu(), varg, dout.cpu(), n_sink=n_sink, window=w, scale=scale, block=block,
                                     out=out.cpu(), lse=lse.cpu())
    if alias:
        rk = rk.copy()
        rk[..., :d_v] += rv
    for name, g, r in [("dq", dq, rq), ("dk", dk, rk)] + ([] if alias else [("dv", dv, rv)]):
        gg = g.double().cpu().numpy()
        assert np.isfinite(gg).all(), f"{label}: {name} has non-finite or unwritten elements"
        err = np.abs(gg - r)
        over = float((err - grad_tolerance_f32(r)).max())
        print(f"[parity] {label}: {name} max|err|={err.max():.3e} max|ref|={np.abs(r).max():.3e}", flush=True)
        assert over <= 0.0, f"{label}: {name} error exceeds its bound by {over} (max error {err.max()})"


def run_backward(q, k, v, out, lse, dout, n_sink, window, scale, block=None):
    """HIP backward through the C ABI. Returns (dq, dk, dv); with ``v is k`` dk is the gradient of the
    shared tensor and dv is None. The outputs start as NaN: every element must be written."""
    B, S, Hq, d_qk = q.shape
    Hkv, d_v = k.shape[2], out.shape[3]
    alias = v is k
    nan = float("nan")
    dq = torch.full_like(q, nan)
    dk = torch.full_like(k, nan)
    dv = None if alias else torch.full_like(v, nan)
    if block is None:
        nb = loza.loza_ssa_backward_workspace_bytes(B, Hq, Hkv, S, d_qk, d_v, n_sink, window, alias)
        ws = torch.empty(max(nb, 16), dtype=torch.uint8, device=q.device)
        loza.loza_ssa_backward(q, k, v, out, lse, dout, dq, dk, dv, n_sink, window, scale, ws)
    else:
        nb = loza.loza_ssa_backward_workspace_bytes_blocks(B, Hq, Hkv, S, d_qk, d_v, n_sink, window, block, alias)
        ws = torch.empty(max(nb, 16), dtype=torch.uint8, device=q.device)
        loza.loza_ssa_backward_blocks(q, k, v, out, lse, dout, dq, dk, dv, n_sink, window, block, scale, ws)
    torch.cuda.synchronize()
    return dq, dk, dv


# Bound on a gradient element. Every element of a gradient row is a sum of products (weight x vector
# element) whose weights (p, dS) reach the matrix cores rounded to bf16 (relative error 2^-9 each, of
# random sign), so its error is a random sum of the same size as 2^-9 times the root-sum-square of
# the terms -- which is also the typical size of the elements of that row, whether or not the
# element itself happens to be small by cancellation. The bound is therefore GRAD_K of those units
# (rms of the reference row times 2^-9), plus the rounding of the result, plus a floor for rows whose
# gradient vanishes by cancellation (a query with one live key has dP = D exactly; the kernel forms
# the two 512-term dot products in fp32 in different orders).
# GRAD_K: one rounded factor per term gives an error of standard deviation 0.58 units (uniform
# rounding error of relative half-width 2^-9 against terms whose root-sum-square is the row's rms x
# sqrt(width)); a term of dK or dQ carries two rounded factors (p inside dS, and dS itself) and the
# rounded `out` inside D shifts every dS of a row together: ~1.2 units of standard deviation where the
# row is dominated by few keys. The maximum over the 10^7 .. 10^8 elements of a test sits 5.5 to 6
# standard deviations out, i.e. at 7 units; measured over every case of the suite: 6 .. 11.4 (the
# high end on rows whose weight sits on one or two keys, where the errors of a row do not average).
# 13 leaves 15 % over the largest value seen.
GRAD_K = 13.0
GRAD_FLOOR = 2e-5


def grad_tolerance(ref: np.ndarray) -> np.ndarray:
    row_rms = np.sqrt((ref ** 2).mean(axis=-1, keepdims=True))
    return GRAD_K * 2.0 ** -9 * row_rms + 2.0 ** -9 * np.abs(ref) + GRAD_FLOOR


def compare_backward(q, k, v, out, lse, dout, got, n_sink, window, scale, label="", block=None):
    """Element by element against the oracle's gradient taken from the same stored out and lse."""
    dq, dk, dv = got
    d_v = dout.shape[3]
    alias = v is k
    w = oracle.INT64_MAX if window is None else window
    varg = ("alias", d_v) if alias else v.cpu()
    rq, rk, rv = oracle.ssa_backward(q.cpu(), k.cpu(), varg, dout.cpu(), n_sink=n_sink, window=w, scale=scale, block=block,
                                     out=out.cpu(), lse=lse.cpu())
    if alias:
        rk = rk.copy()
        rk[..., :d_v] += rv
    pairs = [("dq", dq, rq), ("dk", dk, rk)] + ([] if alias else [("dv", dv, rv)])
    worst = {}
    for name, g, r in pairs:
        gg = g.double().cpu().numpy()
        assert np.isfinite(gg).all(), f"{label}: {name} has non-finite or unwritten elements"
        err = np.abs(gg - r)
        over = float((err - grad_tolerance(r)).max())
        worst[name] = float(err.max())
        unit = 2.0 ** -9 * np.sqrt((r ** 2).mean(axis=-1, keepdims=True)) + GRAD_FLOOR
        print(f"[parity] {label}: {name} max|err|={err.max():.3e} max|ref|={np.abs(r).max():.3e} "
              f"rms err={np.sqrt((err ** 2).mean()):.3e} max err in units of 2^-9 row rms={(err / unit).max():.2f} "
              f"(bound {GRAD_K})", flush=True)
        assert over <= 0.0, f"{label}: {name} error exceeds its bound by {over} (max error {err.max()})"
    return worst
