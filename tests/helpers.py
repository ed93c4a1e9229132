"""Shared plumbing of the GPU parity tests: call the HIP path through the C ABI binding, call the
fp64 oracle on the same bits, compare element by element."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2512_23966_amd as loza

# Tolerances (max abs error against the fp64 oracle). bf16 paths: 1e-2 on the output (the bf16
# rounding of an output of magnitude < 4 alone is up to 2^-8 = 3.9e-3), 1e-3 on the fp32
# log-sum-exp; fp32 path: 1e-5 on both.
TOL = {torch.bfloat16: (1e-2, 1e-3), torch.float32: (1e-5, 1e-5)}


def run_prefill(q, k, v, n_sink, window, scale, d_v=None):
    B, S, Hq, _ = q.shape
    d_v = d_v if d_v is not None else v.shape[3]
    out = torch.empty(B, S, Hq, d_v, dtype=q.dtype, device=q.device)
    lse = torch.empty(B, Hq, S, dtype=torch.float32, device=q.device)
    fn = loza.loza_ssa_prefill if q.dtype == torch.bfloat16 else loza.loza_ssa_prefill_f32
    fn(q, k, v, out, lse, n_sink, window, scale)
    torch.cuda.synchronize()
    return out, lse


def run_decode(q, kc, vc, seqlens, n_sink, window, scale, d_v=None):
    B, Hq, _ = q.shape
    _, S_max, Hkv, _ = kc.shape
    d_v = d_v if d_v is not None else vc.shape[3]
    out = torch.empty(B, Hq, d_v, dtype=torch.bfloat16, device=q.device)
    lse = torch.empty(B, Hq, dtype=torch.float32, device=q.device)
    nbytes = loza.loza_ssa_decode_workspace_bytes(B, Hq, Hkv, S_max, d_v, n_sink, window)
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=q.device)
    loza.loza_ssa_decode(q, kc, vc, seqlens, out, lse, n_sink, window, scale, ws)
    torch.cuda.synchronize()
    return out, lse


def oracle_prefill_rows(q, k, v, rb, rh, ri, n_sink, window, scale, d_v):
    """Oracle on the listed (b, h, i) rows, fed with the very bits the GPU tensors hold."""
    idx = (torch.as_tensor(rb, device=q.device), torch.as_tensor(ri, device=q.device), torch.as_tensor(rh, device=q.device))
    q_rows = q[idx].contiguous().cpu()
    varg = ("alias", d_v) if v is k else v.cpu()
    w = oracle.INT64_MAX if window is None else window
    return oracle.ssa_rows(q_rows, k.cpu(), varg, rb, rh, ri, Hq=q.shape[2], n_sink=n_sink, window=w, scale=scale)


def all_rows(B, Hq, S):
    b, h, i = np.meshgrid(np.arange(B), np.arange(Hq), np.arange(S), indexing="ij")
    return b.ravel().astype(np.int64), h.ravel().astype(np.int64), i.ravel().astype(np.int64)


def compare_prefill(q, k, v, out, lse, rb, rh, ri, n_sink, window, scale, label=""):
    d_v = out.shape[3]
    ref_out, ref_lse = oracle_prefill_rows(q, k, v, rb, rh, ri, n_sink, window, scale, d_v)
    dev = q.device
    idx = (torch.as_tensor(rb, device=dev), torch.as_tensor(ri, device=dev), torch.as_tensor(rh, device=dev))
    got_out = out[idx].double().cpu().numpy()
    got_lse = lse[torch.as_tensor(rb, device=dev), torch.as_tensor(rh, device=dev), torch.as_tensor(ri, device=dev)].double().cpu().numpy()
    assert np.isfinite(got_out).all(), f"{label}: non-finite output"
    e_out = float(np.abs(got_out - ref_out).max())
    e_lse = float(np.abs(got_lse - ref_lse).max())
    tol_out, tol_lse = TOL[q.dtype]
    print(f"[parity] {label}: rows={len(rb)} max|out err|={e_out:.3e} (tol {tol_out}) max|lse err|={e_lse:.3e} (tol {tol_lse})", flush=True)
    assert e_out <= tol_out, f"{label}: out error {e_out} > {tol_out}"
    assert e_lse <= tol_lse, f"{label}: lse error {e_lse} > {tol_lse}"
    return e_out, e_lse


def oracle_decode(q, kc, vc, seqlens, rb, rh, n_sink, window, scale, d_v):
    """Oracle for decode rows (b, h): the query sits at position seqlens[b] - 1 of its cache."""
    L = seqlens.cpu().numpy().astype(np.int64)
    ri = L[rb] - 1
    q_rows = q[torch.as_tensor(rb, device=q.device), torch.as_tensor(rh, device=q.device)].contiguous().cpu()
    # NaN-poisoned rows beyond the length must not reach the oracle's arithmetic either: it never
    # touches a dead key, so the cache is passed as is
    varg = ("alias", d_v) if vc is kc else vc.cpu()
    w = oracle.INT64_MAX if window is None else window
    return oracle.ssa_rows(q_rows, kc.cpu(), varg, rb, rh, ri, Hq=q.shape[1], n_sink=n_sink, window=w, scale=scale)


def compare_decode(q, kc, vc, seqlens, out, lse, rb, rh, n_sink, window, scale, label=""):
    d_v = out.shape[2]
    ref_out, ref_lse = oracle_decode(q, kc, vc, seqlens, rb, rh, n_sink, window, scale, d_v)
    dev = q.device
    got_out = out[torch.as_tensor(rb, device=dev), torch.as_tensor(rh, device=dev)].double().cpu().numpy()
    got_lse = lse[torch.as_tensor(rb, device=dev), torch.as_tensor(rh, device=dev)].double().cpu().numpy()
    assert np.isfinite(got_out).all(), f"{label}: non-finite output"
    e_out = float(np.abs(got_out - ref_out).max())
    e_lse = float(np.abs(got_lse - ref_lse).max())
    tol_out, tol_lse = TOL[torch.bfloat16]
    print(f"[parity] {label}: rows={len(rb)} max|out err|={e_out:.3e} (tol {tol_out}) max|lse err|={e_lse:.3e} (tol {tol_lse})", flush=True)
    assert e_out <= tol_out, f"{label}: out error {e_out} > {tol_out}"
    assert e_lse <= tol_lse, f"{label}: lse error {e_lse} > {tol_lse}"
    return e_out, e_lse
