"""ctypes front end of the fp64 CPU oracle (TEST INFRASTRUCTURE, not the product path).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may
import this package.  It marshals arrays into ``ssa_oracle.c`` and holds no arithmetic of the
method itself; the definition it calls follows the paper's Eq. 2 / Eq. 4 (Architecture section).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "ssa_oracle.c"
_LIB = _HERE / "libssa_oracle.so"
_lib = None

INT64_MAX = (1 << 63) - 1


def build(force: bool = False) -> Path:
    """Compile ssa_oracle.c with gcc (plain C11, -O2, no fast-math)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", str(_LIB), str(_SRC), "-lm", "-lpthread"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(str(_LIB))
        i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        lib.oracle_ssa_rows.restype = ci
        lib.oracle_ssa_rows.argtypes = [vp, vp, vp, ci, i64, vp, vp, vp, ci, ci, ci, i64, ci, ci,
                                        i64, i64, i64, i64, ctypes.c_double, vp, vp, vp, ci]
        lib.oracle_ssa_live_mask.restype = ci
        lib.oracle_ssa_live_mask.argtypes = [i64, i64, i64, i64, vp]
        lib.oracle_ssa_count_pairs.restype = i64
        lib.oracle_ssa_count_pairs.argtypes = [i64, i64, i64]
        lib.oracle_ssa_rows_blocks.restype = ci
        lib.oracle_ssa_rows_blocks.argtypes = [vp, vp, vp, ci, i64, vp, vp, vp, ci, ci, ci, i64, ci, ci,
                                               i64, i64, i64, i64, i64, ctypes.c_double, vp, vp, vp, ci]
        lib.oracle_ssa_live_mask_blocks.restype = ci
        lib.oracle_ssa_live_mask_blocks.argtypes = [i64, i64, i64, i64, i64, vp]
        lib.oracle_ssa_count_pairs_blocks.restype = i64
        lib.oracle_ssa_count_pairs_blocks.argtypes = [i64, i64, i64, i64]
        lib.oracle_ssa_backward.restype = ci
        lib.oracle_ssa_backward.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, i64, ci, ci, i64, i64,
                                            i64, i64, i64, ctypes.c_double, vp, vp, vp, vp, vp, ci]
        lib.oracle_ssa_backward_rows.restype = ci
        lib.oracle_ssa_backward_rows.argtypes = [vp, vp, vp, vp, ci, i64, vp, vp, vp, ci, ci, ci, i64, ci, ci, i64, i64,
                                                 i64, i64, i64, ctypes.c_double, vp, vp, vp, vp, vp, ci]
        _lib = lib
    return _lib


def host_threads() -> int:
    """Threads the oracle uses by default: the cores this process may run on."""
    try:
        return max(1, len(os.sched_getaffinity(0)))
    except AttributeError:  # pragma: no cover
        return max(1, os.cpu_count() or 1)


def as_oracle_array(t):
    """torch tensor / numpy array -> contiguous numpy array the oracle reads (float32, or uint16
    holding bf16 bit patterns).  The bits are passed through unchanged."""
    if isinstance(t, np.ndarray):
        if t.dtype not in (np.float32, np.uint16):
            raise TypeError(f"oracle reads float32 or bf16-as-uint16, got {t.dtype}")
        return np.ascontiguousarray(t)
    import torch
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.float32:
        return t.numpy()
    raise TypeError(f"oracle reads float32 or bfloat16, got {t.dtype}")


def _dtype_code(a: np.ndarray) -> int:
    return 0 if a.dtype == np.float32 else 1


def ssa_rows(q_rows, k, v, row_b, row_h, row_i, *, Hq, n_sink, window, scale,
             want_weights=False, n_threads=None, block=None):
    """SSA (Eq. 4) for the listed query rows.

    ``block=None``: token-granular pattern, ``n_sink`` and ``window`` in tokens. ``block=b``: the
    paper's block-granular pattern, ``n_sink`` = number of sink blocks, ``window`` = number of local
    blocks (the query's own block counted), blocks of ``b`` tokens.

    q_rows [n, d_qk]; k [B, S, Hkv, d_qk]; v [B, S, Hkv, d_v], or ``v=("alias", d_v)`` when the
    values are the first ``d_v`` columns of the key rows (absorbed MLA: one latent serves both).
    Returns (out [n, d_v] float64, lse [n] float64[, weights [n, S] float64]).
    """
    lib = _load()
    qa = as_oracle_array(q_rows)
    ka = as_oracle_array(k)
    if isinstance(v, tuple) and v[0] == "alias":
        va, d_v, v_stride = ka, int(v[1]), ka.shape[3]
    else:
        va = as_oracle_array(v)
        d_v, v_stride = va.shape[3], va.shape[3]
    if not (qa.dtype == ka.dtype == va.dtype):
        raise TypeError("q, k, v must share a dtype")
    B, S, Hkv, k_stride = ka.shape
    n, d_qk = qa.shape
    rb = np.ascontiguousarray(row_b, dtype=np.int64)
    rh = np.ascontiguousarray(row_h, dtype=np.int64)
    ri = np.ascontiguousarray(row_i, dtype=np.int64)
    assert rb.shape == rh.shape == ri.shape == (n,)
    out = np.empty((n, d_v), dtype=np.float64)
    lse = np.empty((n,), dtype=np.float64)
    w = np.zeros((n, S), dtype=np.float64) if want_weights else None
    window = min(int(window), INT64_MAX)
    head = (qa.ctypes.data, ka.ctypes.data, va.ctypes.data, _dtype_code(qa), n,
            rb.ctypes.data, rh.ctypes.data, ri.ctypes.data, B, int(Hq), Hkv, S, d_qk, d_v, k_stride, v_stride)
    tail = (float(scale), out.ctypes.data, lse.ctypes.data, w.ctypes.data if w is not None else None,
            int(n_threads or host_threads()))
    if block is None:
        rc = lib.oracle_ssa_rows(*head, int(n_sink), window, *tail)
    else:
        rc = lib.oracle_ssa_rows_blocks(*head, int(n_sink), window, int(block), *tail)
    if rc != 0:
        raise RuntimeError(f"oracle_ssa_rows failed with code {rc}")
    return (out, lse, w) if want_weights else (out, lse)


def live_mask(i, S, n_sink, window) -> np.ndarray:
    """0/1 vector over keys 0..S-1: which keys query i sees."""
    lib = _load()
    m = np.zeros((S,), dtype=np.uint8)
    rc = lib.oracle_ssa_live_mask(int(i), int(S), int(n_sink), min(int(window), INT64_MAX), m.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"oracle_ssa_live_mask failed with code {rc}")
    return m


def count_pairs(S, n_sink, window) -> int:
    """Live (query, key) pairs of a length-S causal prefill, counted one by one."""
    return int(_load().oracle_ssa_count_pairs(int(S), int(n_sink), min(int(window), INT64_MAX)))


def live_mask_blocks(i, S, sink_blocks, local_blocks, block) -> np.ndarray:
    """0/1 vector over keys 0..S-1: which keys query i sees under the block-granular pattern."""
    m = np.zeros((S,), dtype=np.uint8)
    rc = _load().oracle_ssa_live_mask_blocks(int(i), int(S), int(sink_blocks), min(int(local_blocks), INT64_MAX),
                                             int(block), m.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"oracle_ssa_live_mask_blocks failed with code {rc}")
    return m


def count_pairs_blocks(S, sink_blocks, local_blocks, block) -> int:
    """Live (query, key) pairs of a length-S causal prefill under the block-granular pattern."""
    return int(_load().oracle_ssa_count_pairs_blocks(int(S), int(sink_blocks), min(int(local_blocks), INT64_MAX),
                                                     int(block)))


def calibration_rows(q_rows, k, v, row_b, row_h, row_i, *, Hq, sink_blocks, local_blocks, block, alpha, scale,
                     n_threads=None):
    """Calibration forward of the paper (Architecture section, Eq. 3) for the listed rows:
    ``alpha * O + (1 - alpha) * O'`` with O the full causal attention output and O' the streaming
    sparse one (block-granular pattern). Returns (blend, o_full, o_sparse, lse_full, lse_sparse)."""
    o_full, lse_full = ssa_rows(q_rows, k, v, row_b, row_h, row_i, Hq=Hq, n_sink=0, window=INT64_MAX, scale=scale,
                                n_threads=n_threads)
    o_sparse, lse_sparse = ssa_rows(q_rows, k, v, row_b, row_h, row_i, Hq=Hq, n_sink=sink_blocks, window=local_blocks,
                                    block=block, scale=scale, n_threads=n_threads)
    a = float(alpha)
    return a * o_full + (1.0 - a) * o_sparse, o_full, o_sparse, lse_full, lse_sparse


def calibration_alpha_grad(dout, o_full, o_sparse) -> float:
    """Derivative of ``sum(dout * (alpha * O + (1 - alpha) * O'))`` with respect to alpha (the blend of
    the Architecture section, Eq. 3): ``sum(dout * (O - O'))``, in float64."""
    def widen(x):
        if isinstance(x, np.ndarray) and x.dtype == np.float64:
            return x
        a = as_oracle_array(x)
        if a.dtype == np.uint16:  # bf16 bit patterns: exact in float32
            a = (a.astype(np.uint32) << 16).view(np.float32)
        return a.astype(np.float64)
    d, a, s = widen(dout), widen(o_full), widen(o_sparse)
    return float(np.sum(d * (a - s)))


def ssa_backward(q, k, v, dout, *, n_sink, window, scale, block=None, n_threads=None, out=None, lse=None):
    """Gradient of SSA (Eq. 4) with respect to Q, K and V for the scalar ``sum(dout * O)``.

    q [B, S, Hq, d_qk]; k [B, S, Hkv, d_qk]; v [B, S, Hkv, d_v] or ``("alias", d_v)``; dout
    [B, S, Hq, d_v]. Pattern arguments as in :func:`ssa_rows`. Rows whose ``dout`` is zero
    everywhere are skipped (they contribute exactly nothing). ``out`` [B, S, Hq, d_v] (dtype of q)
    and ``lse`` [B, Hq, S] float32, given together, are what a forward pass stored: D and the weights
    are then taken from them as a training step does, instead of from a forward recomputed here.
    Returns float64 arrays
    (dq [B, S, Hq, d_qk], dk [B, S, Hkv, d_qk], dv [B, S, Hkv, d_v]); with aliased values the
    gradient with respect to the shared tensor is ``dk`` with ``dv`` added to its first d_v columns.
    """
    lib = _load()
    qa, ka, da = as_oracle_array(q), as_oracle_array(k), as_oracle_array(dout)
    if isinstance(v, tuple) and v[0] == "alias":
        va, d_v, v_stride = ka, int(v[1]), ka.shape[3]
    else:
        va = as_oracle_array(v)
        d_v, v_stride = va.shape[3], va.shape[3]
    if not (qa.dtype == ka.dtype == va.dtype == da.dtype):
        raise TypeError("q, k, v, dout must share a dtype")
    B, S, Hkv, k_stride = ka.shape
    _, _, Hq, d_qk = qa.shape
    assert qa.shape == (B, S, Hq, d_qk) and da.shape == (B, S, Hq, d_v)
    oa = la = None
    if (out is None) != (lse is None):
        raise ValueError("out and lse come together")
    if out is not None:
        oa = as_oracle_array(out)
        la = as_oracle_array(lse)
        if oa.dtype != qa.dtype or oa.shape != (B, S, Hq, d_v) or la.dtype != np.float32 or la.shape != (B, Hq, S):
            raise TypeError("out must be [B, S, Hq, d_v] in the dtype of q, lse [B, Hq, S] float32")
    dq = np.empty((B, S, Hq, d_qk), dtype=np.float64)
    dk = np.empty((B, S, Hkv, d_qk), dtype=np.float64)
    dv = np.empty((B, S, Hkv, d_v), dtype=np.float64)
    rc = lib.oracle_ssa_backward(qa.ctypes.data, ka.ctypes.data, va.ctypes.data, da.ctypes.data, _dtype_code(qa),
                                 B, Hq, Hkv, S, d_qk, d_v, k_stride, v_stride,
                                 int(n_sink), min(int(window), INT64_MAX), 0 if block is None else int(block),
                                 float(scale), oa.ctypes.data if oa is not None else None,
                                 la.ctypes.data if la is not None else None,
                                 dq.ctypes.data, dk.ctypes.data, dv.ctypes.data,
                                 int(n_threads or host_threads()))
    if rc != 0:
        raise RuntimeError(f"oracle_ssa_backward failed with code {rc}")
    return dq, dk, dv


def ssa_backward_rows(q_rows, k, v, dout_rows, row_b, row_h, row_i, *, Hq, n_sink, window, scale, block=None,
                      n_threads=None, out_rows=None, lse_rows=None):
    """:func:`ssa_backward` for a dO that is zero outside the listed rows (b, h, i).

    q_rows [n, d_qk], dout_rows [n, d_v] (and, together, out_rows [n, d_v], lse_rows [n] float32).
    Returns (dq_rows [n, d_qk], dk [B, S, Hkv, d_qk], dv [B, S, Hkv, d_v]) as float64.
    """
    lib = _load()
    qa, ka, da = as_oracle_array(q_rows), as_oracle_array(k), as_oracle_array(dout_rows)
    if isinstance(v, tuple) and v[0] == "alias":
        va, d_v, v_stride = ka, int(v[1]), ka.shape[3]
    else:
        va = as_oracle_array(v)
        d_v, v_stride = va.shape[3], va.shape[3]
    if not (qa.dtype == ka.dtype == va.dtype == da.dtype):
        raise TypeError("q_rows, k, v, dout_rows must share a dtype")
    B, S, Hkv, k_stride = ka.shape
    n, d_qk = qa.shape
    rb = np.ascontiguousarray(row_b, dtype=np.int64)
    rh = np.ascontiguousarray(row_h, dtype=np.int64)
    ri = np.ascontiguousarray(row_i, dtype=np.int64)
    assert rb.shape == rh.shape == ri.shape == (n,) and da.shape == (n, d_v)
    oa = la = None
    if (out_rows is None) != (lse_rows is None):
        raise ValueError("out_rows and lse_rows come together")
    if out_rows is not None:
        oa, la = as_oracle_array(out_rows), as_oracle_array(lse_rows)
        if oa.dtype != qa.dtype or oa.shape != (n, d_v) or la.dtype != np.float32 or la.shape != (n,):
            raise TypeError("out_rows must be [n, d_v] in the dtype of q_rows, lse_rows [n] float32")
    dq = np.empty((n, d_qk), dtype=np.float64)
    dk = np.empty((B, S, Hkv, d_qk), dtype=np.float64)
    dv = np.empty((B, S, Hkv, d_v), dtype=np.float64)
    rc = lib.oracle_ssa_backward_rows(qa.ctypes.data, ka.ctypes.data, va.ctypes.data, da.ctypes.data, _dtype_code(qa), n,
                                      rb.ctypes.data, rh.ctypes.data, ri.ctypes.data, B, int(Hq), Hkv, S, d_qk, d_v,
                                      k_stride, v_stride, int(n_sink), min(int(window), INT64_MAX),
                                      0 if block is None else int(block), float(scale),
                                      oa.ctypes.data if oa is not None else None,
                                      la.ctypes.data if la is not None else None,
                                      dq.ctypes.data, dk.ctypes.data, dv.ctypes.data, int(n_threads or host_threads()))
    if rc != 0:
        raise RuntimeError(f"oracle_ssa_backward_rows failed with code {rc}")
    return dq, dk, dv
