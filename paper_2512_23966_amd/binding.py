"""Thin ctypes binding of ``libloza_ssa.so``: argument marshalling only.

Every function has the name and the argument order of its C entry point (``include/loza_ssa.h``).
Tensors are torch tensors that already live on the GPU; nothing is computed here and there is no
fallback: if the shared library is missing, importing a symbol from it raises.
"""
from __future__ import annotations

import ctypes
import os
from pathlib import Path

import torch

_PKG = Path(__file__).resolve().parent
# LOZA_SSA_LIB names another build of the same library (kernel experiments); default: the in-tree one
LIB_PATH = Path(os.environ["LOZA_SSA_LIB"]) if os.environ.get("LOZA_SSA_LIB") else _PKG / "libloza_ssa.so"
_lib = None

LOZA_OK = 0
LOZA_WINDOW_INF = (1 << 63) - 1

EXPORTS = (
    "loza_ssa_prefill", "loza_ssa_prefill_f32", "loza_ssa_decode",
    "loza_ssa_decode_workspace_bytes", "loza_ssa_decode_num_splits",
    "loza_ssa_live_ranges", "loza_ssa_live_pairs", "loza_status_str",
    "loza_ssa_prefill_blocks", "loza_ssa_prefill_blocks_f32", "loza_ssa_decode_blocks",
    "loza_ssa_live_ranges_blocks", "loza_ssa_live_pairs_blocks",
    "loza_ssa_decode_paged", "loza_ssa_decode_paged_blocks",
    "loza_ssa_prefill_calibration_blocks", "loza_ssa_calibration_workspace_bytes",
    "loza_ssa_extend", "loza_ssa_extend_blocks", "loza_ssa_extend_paged", "loza_ssa_extend_paged_blocks",
    "loza_ssa_backward", "loza_ssa_backward_blocks",
    "loza_ssa_backward_workspace_bytes", "loza_ssa_backward_workspace_bytes_blocks",
    "loza_ssa_backward_f32", "loza_ssa_backward_blocks_f32",
    "loza_ssa_decode_f32", "loza_ssa_decode_blocks_f32",
    "loza_ssa_calibration_alpha_grad", "loza_ssa_calibration_alpha_grad_workspace_bytes",
    "loza_ssa_decode_static",
)


class LozaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {loza_status_str(status)} ({status})")


def lib() -> ctypes.CDLL:
    """The loaded shared library (built beforehand by ``__graft_entry__.build()``)."""
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`")
        L = ctypes.CDLL(str(LIB_PATH))
        vp, ci, i64, f32, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
        L.loza_ssa_prefill.restype = ci
        L.loza_ssa_prefill.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, i64, ci, ci, i64, i64, f32, vp]
        L.loza_ssa_prefill_f32.restype = ci
        L.loza_ssa_prefill_f32.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, i64, ci, ci, i64, i64, f32, vp]
        L.loza_ssa_decode.restype = ci
        L.loza_ssa_decode.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, i64, ci, ci, i64, i64, f32, vp, sz, vp]
        L.loza_ssa_decode_static.restype = ci
        L.loza_ssa_decode_static.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, i64, ci, ci, i64, i64, f32, vp]
        L.loza_ssa_decode_workspace_bytes.restype = sz
        L.loza_ssa_decode_workspace_bytes.argtypes = [ci, ci, ci, i64, ci, i64, i64]
        L.loza_ssa_decode_num_splits.restype = ci
        L.loza_ssa_decode_num_splits.argtypes = [ci, ci, ci, i64, i64, i64]
        L.loza_ssa_live_ranges.restype = ci
        L.loza_ssa_live_ranges.argtypes = [i64, i64, i64, ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.POINTER(i64)]
        L.loza_ssa_live_pairs.restype = i64
        L.loza_ssa_live_pairs.argtypes = [i64, i64, i64]
        L.loza_ssa_prefill_blocks.restype = ci
        L.loza_ssa_prefill_blocks.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, i64, ci, ci, i64, i64, i64, f32, vp]
        L.loza_ssa_prefill_blocks_f32.restype = ci
        L.loza_ssa_prefill_blocks_f32.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, i64, ci, ci, i64, i64, i64, f32, vp]
        L.loza_ssa_decode_blocks.restype = ci
        L.loza_ssa_decode_blocks.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, i64, ci, ci, i64, i64, i64, f32, vp, sz, vp]
        L.loza_ssa_live_ranges_blocks.restype = ci
        L.loza_ssa_live_ranges_blocks.argtypes = [i64, i64, i64, i64, ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.POINTER(i64)]
        L.loza_ssa_live_pairs_blocks.restype = i64
        L.loza_ssa_live_pairs_blocks.argtypes = [i64, i64, i64, i64]
        L.loza_ssa_decode_paged.restype = ci
        L.loza_ssa_decode_paged.argtypes = [vp, vp, vp, vp, vp, vp, vp, ci, ci, ci, i64, ci, ci, ci, ci, i64, i64, f32, vp, sz, vp]
        L.loza_ssa_decode_paged_blocks.restype = ci
        L.loza_ssa_decode_paged_blocks.argtypes = [vp, vp, vp, vp, vp, vp, vp, ci, ci, ci, i64, ci, ci, ci, ci, i64, i64, i64, f32, vp, sz, vp]
        L.loza_ssa_prefill_calibration_blocks.restype = ci
        L.loza_ssa_prefill_calibration_blocks.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, ci, ci, ci, i64, ci, ci,
                                                          i64, i64, i64, f32, f32, vp, sz, vp]
        L.loza_ssa_calibration_workspace_bytes.restype = sz
        L.loza_ssa_calibration_workspace_bytes.argtypes = [ci, ci, i64, ci]
        L.loza_ssa_extend.restype = ci
        L.loza_ssa_extend.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, i64, ci, ci, ci, i64, i64, f32, vp]
        L.loza_ssa_extend_blocks.restype = ci
        L.loza_ssa_extend_blocks.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, i64, ci, ci, ci, i64, i64, i64, f32, vp]
        L.loza_ssa_extend_paged.restype = ci
        L.loza_ssa_extend_paged.argtypes = [vp, vp, vp, vp, vp, vp, vp, ci, ci, ci, i64, ci, ci, ci, ci, ci, i64, i64, f32, vp]
        L.loza_ssa_extend_paged_blocks.restype = ci
        L.loza_ssa_extend_paged_blocks.argtypes = [vp, vp, vp, vp, vp, vp, vp, ci, ci, ci, i64, ci, ci, ci, ci, ci, i64, i64, i64, f32, vp]
        L.loza_ssa_backward.restype = ci
        L.loza_ssa_backward.argtypes = [vp] * 9 + [ci, ci, ci, i64, ci, ci, i64, i64, f32, vp, sz, vp]
        L.loza_ssa_backward_blocks.restype = ci
        L.loza_ssa_backward_blocks.argtypes = [vp] * 9 + [ci, ci, ci, i64, ci, ci, i64, i64, i64, f32, vp, sz, vp]
        L.loza_ssa_calibration_alpha_grad.restype = ci
        L.loza_ssa_calibration_alpha_grad.argtypes = [vp, vp, vp, vp, i64, vp, sz, vp]
        L.loza_ssa_calibration_alpha_grad_workspace_bytes.restype = sz
        L.loza_ssa_calibration_alpha_grad_workspace_bytes.argtypes = [i64]
        L.loza_ssa_decode_f32.restype = ci
        L.loza_ssa_decode_f32.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, i64, ci, ci, i64, i64, f32, vp]
        L.loza_ssa_decode_blocks_f32.restype = ci
        L.loza_ssa_decode_blocks_f32.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, i64, ci, ci, i64, i64, i64, f32, vp]
        L.loza_ssa_backward_f32.restype = ci
        L.loza_ssa_backward_f32.argtypes = [vp] * 9 + [ci, ci, ci, i64, ci, ci, i64, i64, f32, vp]
        L.loza_ssa_backward_blocks_f32.restype = ci
        L.loza_ssa_backward_blocks_f32.argtypes = [vp] * 9 + [ci, ci, ci, i64, ci, ci, i64, i64, i64, f32, vp]
        L.loza_ssa_backward_workspace_bytes.restype = sz
        L.loza_ssa_backward_workspace_bytes.argtypes = [ci, ci, ci, i64, ci, ci, i64, i64, ci]
        L.loza_ssa_backward_workspace_bytes_blocks.restype = sz
        L.loza_ssa_backward_workspace_bytes_blocks.argtypes = [ci, ci, ci, i64, ci, ci, i64, i64, i64, ci]
        L.loza_status_str.restype = ctypes.c_char_p
        L.loza_status_str.argtypes = [ci]
        _lib = L
    return _lib


def _win(window) -> int:
    return LOZA_WINDOW_INF if window is None else min(int(window), LOZA_WINDOW_INF)


def _dev_ptr(t: torch.Tensor, dtype, name: str) -> int:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a tensor on the GPU")
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def loza_status_str(status: int) -> str:
    return lib().loza_status_str(int(status)).decode()


def loza_ssa_live_ranges(i: int, n_sink: int, window):
    """(sink_end, win_begin, win_end): live(i) = [0, sink_end) U [win_begin, win_end). Host only."""
    a, b, c = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    rc = lib().loza_ssa_live_ranges(int(i), int(n_sink), _win(window), ctypes.byref(a), ctypes.byref(b), ctypes.byref(c))
    if rc != LOZA_OK:
        raise LozaError(rc, "loza_ssa_live_ranges")
    return a.value, b.value, c.value


def loza_ssa_live_pairs(S: int, n_sink: int, window) -> int:
    return int(lib().loza_ssa_live_pairs(int(S), int(n_sink), _win(window)))


def _prefill_common(fn_name, dtype, q, k, v, out, lse, pattern, scale, stream):
    B, S, Hq, d_qk = q.shape
    Hkv = k.shape[2]
    d_v = out.shape[3]
    if k.shape != (B, S, Hkv, d_qk) or out.shape != (B, S, Hq, d_v) or lse.shape != (B, Hq, S):
        raise ValueError("shape mismatch between q, k, out, lse")
    if v is not k and v.shape != (B, S, Hkv, d_v):
        raise ValueError("v must be [B, S, Hkv, d_v] (or the very tensor passed as k)")
    qp, kp = _dev_ptr(q, dtype, "q"), _dev_ptr(k, dtype, "k")
    vp = kp if v is k else _dev_ptr(v, dtype, "v")
    rc = getattr(lib(), fn_name)(qp, kp, vp, _dev_ptr(out, dtype, "out"), _dev_ptr(lse, torch.float32, "lse"),
                                 B, Hq, Hkv, S, d_qk, d_v, *pattern, float(scale), _stream(stream))
    if rc != LOZA_OK:
        raise LozaError(rc, fn_name)


def loza_ssa_prefill(q, k, v, out, lse, n_sink, window, scale, stream=None):
    """bf16 SSA prefill. q [B,S,Hq,d_qk], k [B,S,Hkv,d_qk], v [B,S,Hkv,d_v] or ``v is k`` (absorbed
    MLA: values are the first d_v columns of k), out [B,S,Hq,d_v] bf16, lse [B,Hq,S] fp32.
    ``window=None`` means infinity (full causal attention)."""
    _prefill_common("loza_ssa_prefill", torch.bfloat16, q, k, v, out, lse, (int(n_sink), _win(window)), scale, stream)


def loza_ssa_prefill_f32(q, k, v, out, lse, n_sink, window, scale, stream=None):
    """fp32 twin of :func:`loza_ssa_prefill`."""
    _prefill_common("loza_ssa_prefill_f32", torch.float32, q, k, v, out, lse, (int(n_sink), _win(window)), scale, stream)


def loza_ssa_prefill_blocks(q, k, v, out, lse, sink_blocks, local_blocks, block, scale, stream=None):
    """bf16 SSA prefill under the block-granular pattern (sink blocks, local blocks, block size)."""
    _prefill_common("loza_ssa_prefill_blocks", torch.bfloat16, q, k, v, out, lse,
                    (int(sink_blocks), _win(local_blocks), int(block)), scale, stream)


def loza_ssa_prefill_blocks_f32(q, k, v, out, lse, sink_blocks, local_blocks, block, scale, stream=None):
    """fp32 twin of :func:`loza_ssa_prefill_blocks`."""
    _prefill_common("loza_ssa_prefill_blocks_f32", torch.float32, q, k, v, out, lse,
                    (int(sink_blocks), _win(local_blocks), int(block)), scale, stream)


def loza_ssa_live_ranges_blocks(i: int, sink_blocks: int, local_blocks, block: int):
    """(sink_end, win_begin, win_end) of query i under the block-granular pattern. Host only."""
    a, b, c = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    rc = lib().loza_ssa_live_ranges_blocks(int(i), int(sink_blocks), _win(local_blocks), int(block),
                                           ctypes.byref(a), ctypes.byref(b), ctypes.byref(c))
    if rc != LOZA_OK:
        raise LozaError(rc, "loza_ssa_live_ranges_blocks")
    return a.value, b.value, c.value


def loza_ssa_live_pairs_blocks(S: int, sink_blocks: int, local_blocks, block: int) -> int:
    return int(lib().loza_ssa_live_pairs_blocks(int(S), int(sink_blocks), _win(local_blocks), int(block)))


def loza_ssa_decode_num_splits(B, Hq, Hkv, S_max, n_sink, window) -> int:
    return int(lib().loza_ssa_decode_num_splits(B, Hq, Hkv, int(S_max), int(n_sink), _win(window)))


def loza_ssa_decode_workspace_bytes(B, Hq, Hkv, S_max, d_v, n_sink, window) -> int:
    return int(lib().loza_ssa_decode_workspace_bytes(B, Hq, Hkv, int(S_max), d_v, int(n_sink), _win(window)))


def _decode_common(fn_name, q, kcache, vcache, seqlens, out, lse, pattern, scale, workspace, stream):
    """bf16 SSA decode. q [B,Hq,d_qk], kcache [B,S_max,Hkv,d_qk], vcache [B,S_max,Hkv,d_v] or
    ``vcache is kcache``, seqlens [B] int32 on the GPU, out [B,Hq,d_v] bf16, lse [B,Hq] fp32,
    workspace: uint8 GPU tensor of at least ``loza_ssa_decode_workspace_bytes`` bytes."""
    B, Hq, d_qk = q.shape
    _, S_max, Hkv, _ = kcache.shape
    d_v = out.shape[2]
    if kcache.shape != (B, S_max, Hkv, d_qk) or out.shape != (B, Hq, d_v) or lse.shape != (B, Hq) or seqlens.shape != (B,):
        raise ValueError("shape mismatch between q, kcache, seqlens, out, lse")
    if vcache is not kcache and vcache.shape != (B, S_max, Hkv, d_v):
        raise ValueError("vcache must be [B, S_max, Hkv, d_v] (or the very tensor passed as kcache)")
    bf = torch.bfloat16
    qp, kp = _dev_ptr(q, bf, "q"), _dev_ptr(kcache, bf, "kcache")
    vp = kp if vcache is kcache else _dev_ptr(vcache, bf, "vcache")
    wp = _dev_ptr(workspace, torch.uint8, "workspace")
    rc = getattr(lib(), fn_name)(qp, kp, vp, _dev_ptr(seqlens, torch.int32, "seqlens"), _dev_ptr(out, bf, "out"),
                                 _dev_ptr(lse, torch.float32, "lse"), B, Hq, Hkv, S_max, d_qk, d_v,
                                 *pattern, float(scale), wp, workspace.numel(), _stream(stream))
    if rc != LOZA_OK:
        raise LozaError(rc, fn_name)


def loza_ssa_decode(q, kcache, vcache, seqlens, out, lse, n_sink, window, scale, workspace, stream=None):
    """bf16 SSA decode (token-granular pattern); tensors as in :func:`_decode_common`."""
    _decode_common("loza_ssa_decode", q, kcache, vcache, seqlens, out, lse, (int(n_sink), _win(window)), scale,
                   workspace, stream)


LOZA_DECODE_STATIC_BYTES = 40 << 20


def loza_ssa_decode_static(q, kcache, vcache, seqlens, out, lse, n_sink, window, scale, stream=None):
    """:func:`loza_ssa_decode` without a workspace argument: the library's own static device buffer
    holds the partial results (sizes beyond ``LOZA_DECODE_STATIC_BYTES`` are rejected)."""
    B, Hq, d_qk = q.shape
    _, S_max, Hkv, _ = kcache.shape
    d_v = out.shape[2]
    if kcache.shape != (B, S_max, Hkv, d_qk) or out.shape != (B, Hq, d_v) or lse.shape != (B, Hq) or seqlens.shape != (B,):
        raise ValueError("shape mismatch between q, kcache, seqlens, out, lse")
    if vcache is not kcache and vcache.shape != (B, S_max, Hkv, d_v):
        raise ValueError("vcache must be [B, S_max, Hkv, d_v] (or the very tensor passed as kcache)")
    bf = torch.bfloat16
    qp, kp = _dev_ptr(q, bf, "q"), _dev_ptr(kcache, bf, "kcache")
    vp = kp if vcache is kcache else _dev_ptr(vcache, bf, "vcache")
    rc = lib().loza_ssa_decode_static(qp, kp, vp, _dev_ptr(seqlens, torch.int32, "seqlens"), _dev_ptr(out, bf, "out"),
                                      _dev_ptr(lse, torch.float32, "lse"), B, Hq, Hkv, S_max, d_qk, d_v,
                                      int(n_sink), _win(window), float(scale), _stream(stream))
    if rc != LOZA_OK:
        raise LozaError(rc, "loza_ssa_decode_static")


def loza_ssa_decode_blocks(q, kcache, vcache, seqlens, out, lse, sink_blocks, local_blocks, block, scale, workspace,
                           stream=None):
    """bf16 SSA decode under the block-granular pattern; the workspace is sized by
    ``loza_ssa_decode_workspace_bytes(..., sink_blocks * block, local_blocks * block)``."""
    _decode_common("loza_ssa_decode_blocks", q, kcache, vcache, seqlens, out, lse,
                   (int(sink_blocks), _win(local_blocks), int(block)), scale, workspace, stream)


def _decode_f32_common(fn_name, q, kcache, vcache, seqlens, out, lse, pattern, scale, stream):
    """fp32 SSA decode: the tensors of :func:`_decode_common` with float32 elements, no workspace."""
    B, Hq, d_qk = q.shape
    _, S_max, Hkv, _ = kcache.shape
    d_v = out.shape[2]
    if kcache.shape != (B, S_max, Hkv, d_qk) or out.shape != (B, Hq, d_v) or lse.shape != (B, Hq) or seqlens.shape != (B,):
        raise ValueError("shape mismatch between q, kcache, seqlens, out, lse")
    if vcache is not kcache and vcache.shape != (B, S_max, Hkv, d_v):
        raise ValueError("vcache must be [B, S_max, Hkv, d_v] (or the very tensor passed as kcache)")
    f32 = torch.float32
    qp, kp = _dev_ptr(q, f32, "q"), _dev_ptr(kcache, f32, "kcache")
    vp = kp if vcache is kcache else _dev_ptr(vcache, f32, "vcache")
    rc = getattr(lib(), fn_name)(qp, kp, vp, _dev_ptr(seqlens, torch.int32, "seqlens"), _dev_ptr(out, f32, "out"),
                                 _dev_ptr(lse, f32, "lse"), B, Hq, Hkv, S_max, d_qk, d_v, *pattern, float(scale), _stream(stream))
    if rc != LOZA_OK:
        raise LozaError(rc, fn_name)


def loza_ssa_decode_f32(q, kcache, vcache, seqlens, out, lse, n_sink, window, scale, stream=None):
    """fp32 twin of :func:`loza_ssa_decode` (no workspace)."""
    _decode_f32_common("loza_ssa_decode_f32", q, kcache, vcache, seqlens, out, lse, (int(n_sink), _win(window)), scale, stream)


def loza_ssa_decode_blocks_f32(q, kcache, vcache, seqlens, out, lse, sink_blocks, local_blocks, block, scale, stream=None):
    """fp32 twin of :func:`loza_ssa_decode_blocks` (no workspace)."""
    _decode_f32_common("loza_ssa_decode_blocks_f32", q, kcache, vcache, seqlens, out, lse,
                       (int(sink_blocks), _win(local_blocks), int(block)), scale, stream)


def _decode_paged_common(fn_name, q, k_pages, v_pages, block_table, seqlens, out, lse, pattern, scale, workspace, stream):
    """bf16 SSA decode against a paged cache. q [B,Hq,d_qk], k_pages [num_pages,page_size,Hkv,d_qk],
    v_pages [num_pages,page_size,Hkv,d_v] or ``v_pages is k_pages``, block_table [B,max_pages] int32 and
    seqlens [B] int32 on the GPU, out [B,Hq,d_v] bf16, lse [B,Hq] fp32, workspace uint8."""
    B, Hq, d_qk = q.shape
    num_pages, page_size, Hkv, _ = k_pages.shape
    d_v = out.shape[2]
    if k_pages.shape != (num_pages, page_size, Hkv, d_qk) or out.shape != (B, Hq, d_v) or lse.shape != (B, Hq) \
            or seqlens.shape != (B,) or block_table.dim() != 2 or block_table.shape[0] != B:
        raise ValueError("shape mismatch between q, k_pages, block_table, seqlens, out, lse")
    if v_pages is not k_pages and v_pages.shape != (num_pages, page_size, Hkv, d_v):
        raise ValueError("v_pages must be [num_pages, page_size, Hkv, d_v] (or the very tensor passed as k_pages)")
    bf = torch.bfloat16
    qp, kp = _dev_ptr(q, bf, "q"), _dev_ptr(k_pages, bf, "k_pages")
    vp = kp if v_pages is k_pages else _dev_ptr(v_pages, bf, "v_pages")
    rc = getattr(lib(), fn_name)(qp, kp, vp, _dev_ptr(block_table, torch.int32, "block_table"),
                                 _dev_ptr(seqlens, torch.int32, "seqlens"), _dev_ptr(out, bf, "out"),
                                 _dev_ptr(lse, torch.float32, "lse"), B, Hq, Hkv, num_pages, page_size,
                                 block_table.shape[1], d_qk, d_v, *pattern, float(scale),
                                 _dev_ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream))
    if rc != LOZA_OK:
        raise LozaError(rc, fn_name)


def loza_ssa_decode_paged(q, k_pages, v_pages, block_table, seqlens, out, lse, n_sink, window, scale, workspace,
                          stream=None):
    """Paged-cache decode, token-granular pattern; tensors as in :func:`_decode_paged_common`."""
    _decode_paged_common("loza_ssa_decode_paged", q, k_pages, v_pages, block_table, seqlens, out, lse,
                         (int(n_sink), _win(window)), scale, workspace, stream)


def loza_ssa_decode_paged_blocks(q, k_pages, v_pages, block_table, seqlens, out, lse, sink_blocks, local_blocks, block,
                                 scale, workspace, stream=None):
    """Paged-cache decode, block-granular pattern."""
    _decode_paged_common("loza_ssa_decode_paged_blocks", q, k_pages, v_pages, block_table, seqlens, out, lse,
                         (int(sink_blocks), _win(local_blocks), int(block)), scale, workspace, stream)


def loza_ssa_calibration_workspace_bytes(B, Hq, S, d_v) -> int:
    return int(lib().loza_ssa_calibration_workspace_bytes(B, Hq, int(S), d_v))


def loza_ssa_prefill_calibration_blocks(q, k, v, out, out_full, out_sparse, lse_full, lse_sparse,
                                        sink_blocks, local_blocks, block, alpha, scale, workspace, stream=None):
    """Calibration forward: out = alpha * O_full + (1 - alpha) * O_sparse (bf16). ``out_full`` / ``out_sparse``
    may be None; lse_full, lse_sparse [B,Hq,S] fp32; workspace uint8 of ``loza_ssa_calibration_workspace_bytes``."""
    B, S, Hq, d_qk = q.shape
    Hkv = k.shape[2]
    d_v = out.shape[3]
    bf = torch.bfloat16
    if k.shape != (B, S, Hkv, d_qk) or out.shape != (B, S, Hq, d_v) or lse_full.shape != (B, Hq, S) or lse_sparse.shape != (B, Hq, S):
        raise ValueError("shape mismatch between q, k, out, lse_full, lse_sparse")
    for t in (out_full, out_sparse):
        if t is not None and t.shape != out.shape:
            raise ValueError("out_full / out_sparse must have the shape of out")
    if v is not k and v.shape != (B, S, Hkv, d_v):
        raise ValueError("v must be [B, S, Hkv, d_v] (or the very tensor passed as k)")
    qp, kp = _dev_ptr(q, bf, "q"), _dev_ptr(k, bf, "k")
    vp = kp if v is k else _dev_ptr(v, bf, "v")
    rc = lib().loza_ssa_prefill_calibration_blocks(
        qp, kp, vp, _dev_ptr(out, bf, "out"),
        None if out_full is None else _dev_ptr(out_full, bf, "out_full"),
        None if out_sparse is None else _dev_ptr(out_sparse, bf, "out_sparse"),
        _dev_ptr(lse_full, torch.float32, "lse_full"), _dev_ptr(lse_sparse, torch.float32, "lse_sparse"),
        B, Hq, Hkv, S, d_qk, d_v, int(sink_blocks), _win(local_blocks), int(block), float(alpha), float(scale),
        _dev_ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream))
    if rc != LOZA_OK:
        raise LozaError(rc, "loza_ssa_prefill_calibration_blocks")


def loza_ssa_calibration_alpha_grad_workspace_bytes(n) -> int:
    return int(lib().loza_ssa_calibration_alpha_grad_workspace_bytes(int(n)))


def loza_ssa_calibration_alpha_grad(dout, out_full, out_sparse, dalpha, workspace, stream=None):
    """d(alpha) of the calibration blend: sum of dout * (out_full - out_sparse). Three bf16 GPU tensors of
    one shape, dalpha a float32 GPU tensor of one element, workspace uint8."""
    if out_full.shape != dout.shape or out_sparse.shape != dout.shape or dalpha.numel() != 1:
        raise ValueError("dout, out_full, out_sparse must share a shape; dalpha holds one element")
    bf = torch.bfloat16
    rc = lib().loza_ssa_calibration_alpha_grad(_dev_ptr(dout, bf, "dout"), _dev_ptr(out_full, bf, "out_full"),
                                               _dev_ptr(out_sparse, bf, "out_sparse"), _dev_ptr(dalpha, torch.float32, "dalpha"),
                                               dout.numel(), _dev_ptr(workspace, torch.uint8, "workspace"), workspace.numel(),
                                               _stream(stream))
    if rc != LOZA_OK:
        raise LozaError(rc, "loza_ssa_calibration_alpha_grad")


def _extend_common(fn_name, q, kcache, vcache, seqlens, out, lse, pattern, scale, stream):
    """bf16 SSA extend. q [B,q_len,Hq,d_qk], kcache [B,S_max,Hkv,d_qk], vcache [B,S_max,Hkv,d_v] or
    ``vcache is kcache``, seqlens [B] int32 on the GPU, out [B,q_len,Hq,d_v] bf16, lse [B,Hq,q_len] fp32."""
    B, q_len, Hq, d_qk = q.shape
    _, S_max, Hkv, _ = kcache.shape
    d_v = out.shape[3]
    if kcache.shape != (B, S_max, Hkv, d_qk) or out.shape != (B, q_len, Hq, d_v) or lse.shape != (B, Hq, q_len) \
            or seqlens.shape != (B,):
        raise ValueError("shape mismatch between q, kcache, seqlens, out, lse")
    if vcache is not kcache and vcache.shape != (B, S_max, Hkv, d_v):
        raise ValueError("vcache must be [B, S_max, Hkv, d_v] (or the very tensor passed as kcache)")
    bf = torch.bfloat16
    qp, kp = _dev_ptr(q, bf, "q"), _dev_ptr(kcache, bf, "kcache")
    vp = kp if vcache is kcache else _dev_ptr(vcache, bf, "vcache")
    rc = getattr(lib(), fn_name)(qp, kp, vp, _dev_ptr(seqlens, torch.int32, "seqlens"), _dev_ptr(out, bf, "out"),
                                 _dev_ptr(lse, torch.float32, "lse"), B, Hq, Hkv, S_max, q_len, d_qk, d_v,
                                 *pattern, float(scale), _stream(stream))
    if rc != LOZA_OK:
        raise LozaError(rc, fn_name)


def loza_ssa_extend(q, kcache, vcache, seqlens, out, lse, n_sink, window, scale, stream=None):
    """q_len new tokens per sequence against its cache, token-granular pattern (see :func:`_extend_common`)."""
    _extend_common("loza_ssa_extend", q, kcache, vcache, seqlens, out, lse, (int(n_sink), _win(window)), scale, stream)


def loza_ssa_extend_blocks(q, kcache, vcache, seqlens, out, lse, sink_blocks, local_blocks, block, scale, stream=None):
    """q_len new tokens per sequence against its cache, block-granular pattern."""
    _extend_common("loza_ssa_extend_blocks", q, kcache, vcache, seqlens, out, lse,
                   (int(sink_blocks), _win(local_blocks), int(block)), scale, stream)


def _extend_paged_common(fn_name, q, k_pages, v_pages, block_table, seqlens, out, lse, pattern, scale, stream):
    """bf16 SSA extend against a paged cache: q [B,q_len,Hq,d_qk], k_pages [num_pages,page_size,Hkv,d_qk],
    v_pages likewise with d_v (or ``v_pages is k_pages``), block_table [B,max_pages] int32, seqlens [B] int32,
    out [B,q_len,Hq,d_v] bf16, lse [B,Hq,q_len] fp32."""
    B, q_len, Hq, d_qk = q.shape
    num_pages, page_size, Hkv, _ = k_pages.shape
    d_v = out.shape[3]
    if k_pages.shape != (num_pages, page_size, Hkv, d_qk) or out.shape != (B, q_len, Hq, d_v) or lse.shape != (B, Hq, q_len) \
            or seqlens.shape != (B,) or block_table.dim() != 2 or block_table.shape[0] != B:
        raise ValueError("shape mismatch between q, k_pages, block_table, seqlens, out, lse")
    if v_pages is not k_pages and v_pages.shape != (num_pages, page_size, Hkv, d_v):
        raise ValueError("v_pages must be [num_pages, page_size, Hkv, d_v] (or the very tensor passed as k_pages)")
    bf = torch.bfloat16
    qp, kp = _dev_ptr(q, bf, "q"), _dev_ptr(k_pages, bf, "k_pages")
    vp = kp if v_pages is k_pages else _dev_ptr(v_pages, bf, "v_pages")
    rc = getattr(lib(), fn_name)(qp, kp, vp, _dev_ptr(block_table, torch.int32, "block_table"),
                                 _dev_ptr(seqlens, torch.int32, "seqlens"), _dev_ptr(out, bf, "out"),
                                 _dev_ptr(lse, torch.float32, "lse"), B, Hq, Hkv, num_pages, page_size,
                                 block_table.shape[1], q_len, d_qk, d_v, *pattern, float(scale), _stream(stream))
    if rc != LOZA_OK:
        raise LozaError(rc, fn_name)


def loza_ssa_extend_paged(q, k_pages, v_pages, block_table, seqlens, out, lse, n_sink, window, scale, stream=None):
    """Extend against a paged cache, token-granular pattern (see :func:`_extend_paged_common`)."""
    _extend_paged_common("loza_ssa_extend_paged", q, k_pages, v_pages, block_table, seqlens, out, lse,
                         (int(n_sink), _win(window)), scale, stream)


def loza_ssa_extend_paged_blocks(q, k_pages, v_pages, block_table, seqlens, out, lse, sink_blocks, local_blocks, block,
                                 scale, stream=None):
    """Extend against a paged cache, block-granular pattern."""
    _extend_paged_common("loza_ssa_extend_paged_blocks", q, k_pages, v_pages, block_table, seqlens, out, lse,
                         (int(sink_blocks), _win(local_blocks), int(block)), scale, stream)


def loza_ssa_backward_workspace_bytes(B, Hq, Hkv, S, d_qk, d_v, n_sink, window, v_aliases_k) -> int:
    return int(lib().loza_ssa_backward_workspace_bytes(B, Hq, Hkv, int(S), d_qk, d_v, int(n_sink), _win(window),
                                                       1 if v_aliases_k else 0))


def loza_ssa_backward_workspace_bytes_blocks(B, Hq, Hkv, S, d_qk, d_v, sink_blocks, local_blocks, block,
                                             v_aliases_k) -> int:
    return int(lib().loza_ssa_backward_workspace_bytes_blocks(B, Hq, Hkv, int(S), d_qk, d_v, int(sink_blocks),
                                                              _win(local_blocks), int(block), 1 if v_aliases_k else 0))


def _backward_common(fn_name, q, k, v, out, lse, dout, dq, dk, dv, pattern, scale, workspace, stream):
    """bf16 SSA backward. q, dq [B,S,Hq,d_qk]; k, dk [B,S,Hkv,d_qk]; v, dv [B,S,Hkv,d_v] (``v is k``:
    dk receives the gradient of the shared tensor, dv is None); out, dout [B,S,Hq,d_v] bf16; lse
    [B,Hq,S] fp32; workspace uint8 of at least ``loza_ssa_backward_workspace_bytes`` bytes."""
    B, S, Hq, d_qk = q.shape
    Hkv = k.shape[2]
    d_v = out.shape[3]
    if k.shape != (B, S, Hkv, d_qk) or out.shape != (B, S, Hq, d_v) or dout.shape != out.shape \
            or lse.shape != (B, Hq, S) or dq.shape != q.shape or dk.shape != k.shape:
        raise ValueError("shape mismatch between q, k, out, lse, dout, dq, dk")
    bf = torch.bfloat16
    kp = _dev_ptr(k, bf, "k")
    if v is k:
        vp, dvp = kp, None
    else:
        if v.shape != (B, S, Hkv, d_v) or dv is None or dv.shape != v.shape:
            raise ValueError("v and dv must be [B, S, Hkv, d_v] (or v the very tensor passed as k)")
        vp, dvp = _dev_ptr(v, bf, "v"), _dev_ptr(dv, bf, "dv")
    rc = getattr(lib(), fn_name)(_dev_ptr(q, bf, "q"), kp, vp, _dev_ptr(out, bf, "out"), _dev_ptr(lse, torch.float32, "lse"),
                                 _dev_ptr(dout, bf, "dout"), _dev_ptr(dq, bf, "dq"), _dev_ptr(dk, bf, "dk"), dvp,
                                 B, Hq, Hkv, S, d_qk, d_v, *pattern, float(scale),
                                 _dev_ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream))
    if rc != LOZA_OK:
        raise LozaError(rc, fn_name)


def _backward_f32_common(fn_name, q, k, v, out, lse, dout, dq, dk, dv, pattern, scale, stream):
    """fp32 SSA backward: the tensors of :func:`_backward_common` with float32 elements, no workspace."""
    B, S, Hq, d_qk = q.shape
    Hkv = k.shape[2]
    d_v = out.shape[3]
    if k.shape != (B, S, Hkv, d_qk) or out.shape != (B, S, Hq, d_v) or dout.shape != out.shape \
            or lse.shape != (B, Hq, S) or dq.shape != q.shape or dk.shape != k.shape:
        raise ValueError("shape mismatch between q, k, out, lse, dout, dq, dk")
    f32 = torch.float32
    kp = _dev_ptr(k, f32, "k")
    if v is k:
        vp, dvp = kp, None
    else:
        if v.shape != (B, S, Hkv, d_v) or dv is None or dv.shape != v.shape:
            raise ValueError("v and dv must be [B, S, Hkv, d_v] (or v the very tensor passed as k)")
        vp, dvp = _dev_ptr(v, f32, "v"), _dev_ptr(dv, f32, "dv")
    rc = getattr(lib(), fn_name)(_dev_ptr(q, f32, "q"), kp, vp, _dev_ptr(out, f32, "out"), _dev_ptr(lse, f32, "lse"),
                                 _dev_ptr(dout, f32, "dout"), _dev_ptr(dq, f32, "dq"), _dev_ptr(dk, f32, "dk"), dvp,
                                 B, Hq, Hkv, S, d_qk, d_v, *pattern, float(scale), _stream(stream))
    if rc != LOZA_OK:
        raise LozaError(rc, fn_name)


def loza_ssa_backward_f32(q, k, v, out, lse, dout, dq, dk, dv, n_sink, window, scale, stream=None):
    """fp32 twin of :func:`loza_ssa_backward`."""
    _backward_f32_common("loza_ssa_backward_f32", q, k, v, out, lse, dout, dq, dk, dv, (int(n_sink), _win(window)), scale, stream)


def loza_ssa_backward_blocks_f32(q, k, v, out, lse, dout, dq, dk, dv, sink_blocks, local_blocks, block, scale, stream=None):
    """fp32 twin of :func:`loza_ssa_backward_blocks`."""
    _backward_f32_common("loza_ssa_backward_blocks_f32", q, k, v, out, lse, dout, dq, dk, dv,
                         (int(sink_blocks), _win(local_blocks), int(block)), scale, stream)


def loza_ssa_backward(q, k, v, out, lse, dout, dq, dk, dv, n_sink, window, scale, workspace, stream=None):
    """Gradients of :func:`loza_ssa_prefill` (token-granular pattern); tensors as in :func:`_backward_common`."""
    _backward_common("loza_ssa_backward", q, k, v, out, lse, dout, dq, dk, dv, (int(n_sink), _win(window)), scale,
                     workspace, stream)


def loza_ssa_backward_blocks(q, k, v, out, lse, dout, dq, dk, dv, sink_blocks, local_blocks, block, scale, workspace,
                             stream=None):
    """Gradients of :func:`loza_ssa_prefill_blocks` (block-granular pattern)."""
    _backward_common("loza_ssa_backward_blocks", q, k, v, out, lse, dout, dq, dk, dv,
                     (int(sink_blocks), _win(local_blocks), int(block)), scale, workspace, stream)
