"""Host side of the C ABI, no GPU needed: the library loads, exports what the header declares,
rejects bad arguments before touching HIP, and its host-only live-set arithmetic agrees with the
oracle's explicit mask."""
import ctypes
import re
from pathlib import Path

import numpy as np
import pytest

import oracle
from paper_2512_23966_amd import binding as B

ROOT = Path(__file__).resolve().parent.parent
HEADER = ROOT / "include" / "loza_ssa.h"
INF = B.LOZA_WINDOW_INF

ERR_NULL, ERR_SHAPE, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP, ERR_ALIGN = -1, -2, -3, -4, -5, -6


def declared_functions():
    """Names of the functions include/loza_ssa.h declares (comments stripped)."""
    text = re.sub(r"/\*.*?\*/", "", HEADER.read_text(), flags=re.S)
    return sorted(set(re.findall(r"\b(loza_\w+)\s*\(", text)))


def test_header_declares_the_binding_exports():
    assert declared_functions() == sorted(B.EXPORTS)


def test_library_exports_every_declared_symbol():
    L = B.lib()
    for name in declared_functions():
        assert hasattr(L, name), name


def test_status_strings_are_distinct():
    names = {B.loza_status_str(s) for s in range(0, -7, -1)}
    assert len(names) == 7
    assert B.loza_status_str(-99)  # unknown codes still give a string


# ---- live ranges and pair counts against the oracle's mask ------------------------------------

@pytest.mark.parametrize("n_sink,window", [(0, 1), (1, 1), (4, 8), (128, 1024), (0, INF), (7, 3), (64, 256), (300, 5)])
def test_live_ranges_match_oracle_mask(n_sink, window):
    S = 700
    w = window if window != INF else oracle.INT64_MAX
    for i in list(range(0, 40)) + [63, 64, 127, 128, 255, 256, 257, 299, 300, 301, 305, 699]:
        se, wb, we = B.loza_ssa_live_ranges(i, n_sink, window)
        assert 0 <= se <= wb <= we == i + 1
        got = np.zeros(S, dtype=bool)
        got[:se] = True
        got[wb:we] = True
        assert np.array_equal(got, oracle.live_mask(i, S, n_sink, w).astype(bool)), (i, se, wb, we)


def test_live_ranges_rejects_bad_arguments():
    L = B.lib()
    a, b, c = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    assert L.loza_ssa_live_ranges(-1, 0, 1, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)) == ERR_SHAPE
    assert L.loza_ssa_live_ranges(0, -1, 1, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)) == ERR_SHAPE
    assert L.loza_ssa_live_ranges(0, 0, 0, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)) == ERR_SHAPE
    assert L.loza_ssa_live_ranges(0, 0, 1, None, ctypes.byref(b), ctypes.byref(c)) == ERR_NULL


@pytest.mark.parametrize("S,n_sink,window", [(1, 0, 1), (700, 4, 8), (700, 0, INF), (1024, 64, 256), (700, 300, 5),
                                             (32768, 128, 4096), (20000, 128, 8192)])
def test_live_pairs_match_oracle_count(S, n_sink, window):
    w = window if window != INF else oracle.INT64_MAX
    assert B.loza_ssa_live_pairs(S, n_sink, window) == oracle.count_pairs(S, n_sink, w)


def test_live_pairs_closed_form_of_the_headline_shape():
    # T = n_sink + window keys once the sequence is longer than that: T(T+1)/2 + (S - T) T
    S, T = 131072, 128 + 8192
    assert B.loza_ssa_live_pairs(S, 128, 8192) == T * (T + 1) // 2 + (S - T) * T


@pytest.mark.parametrize("s,l,b", [(1, 2, 3), (0, 1, 4), (1, 7, 128), (2, 1, 2), (1, 3, 1), (3, 2, 50), (1, 1, 1000), (0, INF, 5)])
def test_block_live_ranges_match_oracle_mask(s, l, b):
    S = 700
    lo = l if l != INF else oracle.INT64_MAX
    for i in list(range(0, 40)) + [63, 64, 127, 128, 255, 256, 257, 383, 384, 511, 512, 699]:
        se, wb, we = B.loza_ssa_live_ranges_blocks(i, s, l, b)
        assert 0 <= se <= wb <= we == i + 1
        got = np.zeros(S, dtype=bool)
        got[:se] = True
        got[wb:we] = True
        assert np.array_equal(got, oracle.live_mask_blocks(i, S, s, lo, b).astype(bool)), (i, se, wb, we)


@pytest.mark.parametrize("S,s,l,b", [(1, 0, 1, 1), (700, 1, 2, 3), (700, 1, 7, 128), (1024, 1, 7, 128), (2500, 1, 7, 128),
                                     (700, 3, 2, 50), (333, 0, 1, 1000), (700, 4, 8, 1), (5000, 2, 3, 128)])
def test_block_live_pairs_match_oracle_count(S, s, l, b):
    assert B.loza_ssa_live_pairs_blocks(S, s, l, b) == oracle.count_pairs_blocks(S, s, l, b)


def test_block_size_one_is_the_token_pattern_on_the_host_too():
    for i in (0, 5, 99, 1000):
        assert B.loza_ssa_live_ranges_blocks(i, 7, 20, 1) == B.loza_ssa_live_ranges(i, 7, 20)
    assert B.loza_ssa_live_pairs_blocks(4000, 7, 20, 1) == B.loza_ssa_live_pairs(4000, 7, 20)


def test_block_entry_points_reject_bad_patterns():
    L = B.lib()
    a, b_, c = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    for s, l, b in ((-1, 1, 2), (0, 0, 2), (1, 1, 0)):
        assert L.loza_ssa_live_ranges_blocks(3, s, l, b, ctypes.byref(a), ctypes.byref(b_), ctypes.byref(c)) == ERR_SHAPE
        assert B.loza_ssa_live_pairs_blocks(10, s, l, b) == -1
        assert L.loza_ssa_prefill_blocks(FAKE, FAKE, FAKE, FAKE, FAKE, 1, 64, 1, 256, 576, 512, s, l, b, 0.07, None) == ERR_SHAPE
        assert L.loza_ssa_prefill_blocks_f32(FAKE, FAKE, FAKE, FAKE, FAKE, 1, 2, 1, 256, 64, 64, s, l, b, 0.07, None) == ERR_SHAPE
        assert L.loza_ssa_decode_blocks(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 2, 64, 1, 4096, 576, 512, s, l, b, 0.07,
                                        FAKE, 1 << 30, None) == ERR_SHAPE
    assert L.loza_ssa_prefill_blocks(None, FAKE, FAKE, FAKE, FAKE, 1, 64, 1, 256, 576, 512, 1, 7, 128, 0.07, None) == ERR_NULL
    assert L.loza_ssa_prefill_blocks(FAKE, FAKE, FAKE + 64, FAKE, FAKE, 1, 64, 1, 256, 96, 96, 1, 7, 128, 0.07, None) == ERR_UNSUPPORTED
    assert L.loza_ssa_decode_blocks(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 2, 64, 1, 4096, 576, 512, 1, 7, 128, 0.07,
                                    FAKE, 15, None) == ERR_WORKSPACE


def _paged(page_size=128, num_pages=100, max_pages=8, table=None, ws_bytes=1 << 30, **kw):
    args = dict(B_=2, Hq=64, Hkv=1, d_qk=576, d_v=512, n_sink=128, window=256, scale=0.07)
    args.update(kw)
    return B.lib().loza_ssa_decode_paged(FAKE, FAKE, FAKE, FAKE if table is None else table, FAKE, FAKE, FAKE,
                                         args["B_"], args["Hq"], args["Hkv"], num_pages, page_size, max_pages,
                                         args["d_qk"], args["d_v"], args["n_sink"], args["window"], args["scale"],
                                         FAKE, ws_bytes, None)


def test_paged_decode_rejects_bad_paging():
    assert _paged(page_size=96) == ERR_SHAPE      # not a power of two
    assert _paged(page_size=16) == ERR_SHAPE      # smaller than a key tile
    assert _paged(num_pages=0) == ERR_SHAPE
    assert _paged(max_pages=0) == ERR_SHAPE
    assert _paged(max_pages=1 << 30) == ERR_SHAPE  # capacity beyond the supported sequence length
    assert _paged(ws_bytes=15) == ERR_WORKSPACE
    assert _paged(window=0) == ERR_SHAPE
    assert _paged(d_qk=80, d_v=80) == ERR_UNSUPPORTED
    assert B.lib().loza_ssa_decode_paged(FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, 2, 64, 1, 100, 128, 8, 576, 512,
                                         128, 256, 0.07, FAKE, 1 << 30, None) == ERR_NULL
    assert B.lib().loza_ssa_decode_paged_blocks(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 2, 64, 1, 100, 128, 8, 576, 512,
                                                1, 0, 128, 0.07, FAKE, 1 << 30, None) == ERR_SHAPE


def test_calibration_workspace_and_validation():
    assert B.loza_ssa_calibration_workspace_bytes(2, 64, 1000, 512) == 2 * 2 * 1000 * 64 * 512 * 4
    assert B.loza_ssa_calibration_workspace_bytes(0, 64, 1000, 512) == 0

    def call(alpha=0.5, out=FAKE, lse_f=FAKE, ws=FAKE, ws_bytes=1 << 40, s=1, l=7, b=128, d_qk=576, d_v=512, v=FAKE):
        return B.lib().loza_ssa_prefill_calibration_blocks(FAKE, FAKE, v, out, None, None, lse_f, FAKE, 1, 64, 1, 256,
                                                           d_qk, d_v, s, l, b, alpha, 0.07, ws, ws_bytes, None)
    assert call(alpha=1.5) == ERR_SHAPE
    assert call(alpha=-0.1) == ERR_SHAPE
    assert call(alpha=float("nan")) == ERR_SHAPE
    assert call(out=None) == ERR_NULL
    assert call(lse_f=None) == ERR_NULL
    assert call(ws=None) == ERR_WORKSPACE
    assert call(ws_bytes=1000) == ERR_WORKSPACE
    assert call(l=0) == ERR_SHAPE
    assert call(d_qk=96, d_v=96, v=FAKE + 64) == ERR_UNSUPPORTED


def test_extend_rejects_bad_arguments():
    def call(q_len=4, sl=FAKE, S_max=4096, window=256, scale=0.07, d_qk=576, d_v=512, v=FAKE):
        return B.lib().loza_ssa_extend(FAKE, FAKE, v, sl, FAKE, FAKE, 2, 64, 1, S_max, q_len, d_qk, d_v, 128, window, scale, None)
    assert call(q_len=0) == ERR_SHAPE
    assert call(q_len=5000) == ERR_SHAPE      # more queries than the cache has rows
    assert call(sl=None) == ERR_NULL
    assert call(sl=FAKE + 2) == ERR_ALIGN
    assert call(window=0) == ERR_SHAPE
    assert call(scale=0.0) == ERR_SHAPE
    assert call(d_qk=96, d_v=96, v=FAKE + 64) == ERR_UNSUPPORTED
    assert B.lib().loza_ssa_extend_blocks(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 2, 64, 1, 4096, 4, 576, 512, 1, 7, 0, 0.07, None) == ERR_SHAPE


def test_extend_paged_rejects_bad_paging():
    def call(page_size=128, num_pages=100, max_pages=8, q_len=4, table=FAKE):
        return B.lib().loza_ssa_extend_paged(FAKE, FAKE, FAKE, table, FAKE, FAKE, FAKE, 2, 64, 1, num_pages, page_size,
                                             max_pages, q_len, 576, 512, 128, 256, 0.07, None)
    assert call(page_size=96) == ERR_SHAPE
    assert call(page_size=16) == ERR_SHAPE
    assert call(num_pages=0) == ERR_SHAPE
    assert call(max_pages=0) == ERR_SHAPE
    assert call(q_len=2000) == ERR_SHAPE       # more queries than the table can hold rows
    assert call(table=None) == ERR_NULL
    assert call(table=FAKE + 2) == ERR_ALIGN


# ---- argument validation: every case returns before the first HIP call --------------------------

FAKE = 0x1000  # aligned, non-null, never dereferenced: validation fails first


def _prefill(fn="loza_ssa_prefill", q=FAKE, k=FAKE, v=FAKE, out=FAKE, lse=FAKE, B_=1, Hq=64, Hkv=1, S=256,
             d_qk=None, d_v=None, n_sink=128, window=64, scale=0.07):
    if d_qk is None:  # a shape the entry point has a kernel for
        d_qk, d_v = (576, 512) if fn == "loza_ssa_prefill" else (64, 64)
    return getattr(B.lib(), fn)(q, k, v, out, lse, B_, Hq, Hkv, S, d_qk, d_v, n_sink, window, scale, None)


@pytest.mark.parametrize("fn", ["loza_ssa_prefill", "loza_ssa_prefill_f32"])
def test_prefill_rejects_null_and_misaligned(fn):
    for name in ("q", "k", "v", "out", "lse"):
        assert _prefill(fn, **{name: None}) == ERR_NULL, name
    for name in ("q", "out"):
        assert _prefill(fn, **{name: FAKE + 2}) == ERR_ALIGN, name
    assert _prefill(fn, k=FAKE + 2, v=FAKE + 2) == ERR_ALIGN


@pytest.mark.parametrize("fn", ["loza_ssa_prefill", "loza_ssa_prefill_f32"])
def test_prefill_rejects_bad_sizes(fn):
    assert _prefill(fn, B_=0) == ERR_SHAPE
    assert _prefill(fn, S=0) == ERR_SHAPE
    assert _prefill(fn, Hq=6, Hkv=4) == ERR_SHAPE
    assert _prefill(fn, n_sink=-1) == ERR_SHAPE
    assert _prefill(fn, window=0) == ERR_SHAPE
    assert _prefill(fn, scale=float("nan")) == ERR_SHAPE
    assert _prefill(fn, scale=float("inf")) == ERR_SHAPE
    assert _prefill(fn, S=1 << 31) == ERR_SHAPE


def test_bf16_prefill_rejects_non_positive_scale_and_unbuilt_shapes():
    assert _prefill(scale=0.0) == ERR_SHAPE
    assert _prefill(scale=-0.1) == ERR_SHAPE
    assert _prefill(d_qk=96, d_v=96, v=FAKE + 64) == ERR_UNSUPPORTED
    assert _prefill(d_qk=576, d_v=512, v=FAKE + 64) == ERR_UNSUPPORTED  # the MLA shape needs v == k
    assert _prefill(d_qk=64, d_v=128) == ERR_SHAPE                      # v == k needs d_v <= d_qk


def test_f32_prefill_rejects_wide_heads():
    assert _prefill("loza_ssa_prefill_f32", d_qk=257, d_v=64, v=FAKE + 64) == ERR_UNSUPPORTED


def _decode(q=FAKE, kc=FAKE, vc=FAKE, sl=FAKE, out=FAKE, lse=FAKE, B_=4, Hq=64, Hkv=1, S_max=4096, d_qk=576, d_v=512,
            n_sink=128, window=1024, scale=0.07, ws=FAKE, ws_bytes=None):
    if ws_bytes is None:
        ws_bytes = B.loza_ssa_decode_workspace_bytes(B_, Hq, Hkv, S_max, d_v, n_sink, window)
    return B.lib().loza_ssa_decode(q, kc, vc, sl, out, lse, B_, Hq, Hkv, S_max, d_qk, d_v, n_sink, window, scale,
                                   ws, ws_bytes, None)


def test_decode_rejects_bad_arguments():
    for name in ("q", "kc", "vc", "sl", "out", "lse"):
        assert _decode(**{name: None}) == ERR_NULL, name
    assert _decode(ws=None) == ERR_WORKSPACE
    assert _decode(ws_bytes=15) == ERR_WORKSPACE
    assert _decode(q=FAKE + 4) == ERR_ALIGN
    assert _decode(window=0) == ERR_SHAPE
    assert _decode(scale=0.0) == ERR_SHAPE
    assert _decode(Hq=65, Hkv=2) == ERR_SHAPE
    assert _decode(d_qk=80, d_v=80, vc=FAKE + 64) == ERR_UNSUPPORTED


def test_decode_split_count_and_workspace_size():
    # enough splits to give each of the 256 compute units a workgroup, never more than key tiles
    assert B.loza_ssa_decode_num_splits(64, 64, 1, 262144, 128, 8192) == 4
    assert B.loza_ssa_decode_num_splits(256, 64, 1, 262144, 128, 8192) == 1
    assert B.loza_ssa_decode_num_splits(1, 64, 1, 64, 0, 64) <= 3
    n = B.loza_ssa_decode_num_splits(3, 32, 4, 10000, 16, 512)
    assert 1 <= n <= 64
    # per (b, query head, split): d_v fp32 of partial output and four floats of softmax state
    assert B.loza_ssa_decode_workspace_bytes(3, 32, 4, 10000, 128, 16, 512) == 3 * 32 * n * (128 + 4) * 4
    assert B.loza_ssa_decode_workspace_bytes(0, 32, 4, 10000, 128, 16, 512) == 0
    assert B.loza_ssa_decode_num_splits(3, 32, 5, 10000, 16, 512) == 0


def test_backward_rejects_bad_arguments_and_sizes_its_workspace():
    big = 1 << 40

    def call(q=FAKE, v=FAKE, dv=None, dout=FAKE, Hq=64, Hkv=1, S=4096, d_qk=576, d_v=512, n_sink=128, window=512,
             scale=0.07, ws=FAKE, ws_bytes=big):
        return B.lib().loza_ssa_backward(q, FAKE, v, FAKE, FAKE, dout, FAKE, FAKE, dv, 1, Hq, Hkv, S, d_qk, d_v,
                                         n_sink, window, scale, ws, ws_bytes, None)
    assert call(q=None) == ERR_NULL and call(dout=None) == ERR_NULL
    assert call(v=FAKE + 64, d_qk=128, d_v=128, dv=None) == ERR_NULL        # separate values need their own dv
    assert call(window=0) == ERR_SHAPE and call(n_sink=-1) == ERR_SHAPE and call(scale=0.0) == ERR_SHAPE
    assert call(d_qk=96, d_v=96) == ERR_UNSUPPORTED
    assert call(Hq=3) == ERR_UNSUPPORTED and call(Hq=48) == ERR_UNSUPPORTED  # heads per group: 2^n <= 32 or 32 n
    assert call(Hq=96) != ERR_UNSUPPORTED
    assert call(ws=None) == ERR_WORKSPACE and call(ws_bytes=16) == ERR_WORKSPACE
    assert call(dout=FAKE + 8) == ERR_ALIGN
    assert B.lib().loza_ssa_backward_blocks(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, 1, 64, 1, 4096, 576, 512,
                                            1, 7, 0, 0.07, FAKE, big, None) == ERR_SHAPE
    # the row statistics (8 bytes per query row, rows padded to 32 per kv head) ...
    assert B.loza_ssa_backward_workspace_bytes(2, 8, 2, 1000, 128, 128, 0, 100, False) == 2 * 2 * 4000 * 8
    # ... plus, with sink keys, fp32 partial sums of the sink key tiles: one per chunk of query rows
    n = B.loza_ssa_backward_workspace_bytes(1, 64, 1, 131072, 576, 512, 128, 8192, True)
    stat = 131072 * 64 * 8
    assert n > stat and (n - stat) % (2 * 64 * 576 * 4) == 0       # two key tiles of 64 keys, 576 columns
    assert B.loza_ssa_backward_workspace_bytes(1, 3, 1, 1000, 128, 128, 0, 100, False) == 0
    assert B.loza_ssa_backward_workspace_bytes_blocks(1, 64, 1, 4096, 576, 512, 1, 7, 0, True) == 0
    assert B.loza_ssa_backward_workspace_bytes_blocks(1, 64, 1, 4096, 576, 512, 1, 7, 128, True) > 0


def test_backward_f32_rejects_bad_arguments():
    def call(q=FAKE, v=FAKE + 64, dv=FAKE, dout=FAKE, Hq=4, Hkv=2, S=100, d_qk=64, d_v=64, n_sink=3, window=10, scale=0.1):
        return B.lib().loza_ssa_backward_f32(q, FAKE, v, FAKE, FAKE, dout, FAKE, FAKE, dv, 1, Hq, Hkv, S, d_qk, d_v,
                                             n_sink, window, scale, None)
    assert call(q=None) == ERR_NULL and call(dout=None) == ERR_NULL
    assert call(dv=None) == ERR_NULL                     # separate values need their own dv
    assert call(v=FAKE, dv=None, d_v=96) == ERR_SHAPE    # aliased values wider than the keys
    assert call(window=0) == ERR_SHAPE and call(n_sink=-1) == ERR_SHAPE and call(Hq=3) == ERR_SHAPE
    assert call(d_qk=257) == ERR_UNSUPPORTED and call(d_v=300) == ERR_UNSUPPORTED
    assert call(dout=FAKE + 4) == ERR_ALIGN
    assert B.lib().loza_ssa_backward_blocks_f32(FAKE, FAKE, FAKE + 64, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1, 4, 2, 100, 64, 64,
                                                1, 7, 0, 0.1, None) == ERR_SHAPE


def test_decode_f32_rejects_bad_arguments():
    def call(q=FAKE, vc=FAKE + 64, lens=FAKE, Hq=4, Hkv=2, S=100, d_qk=64, d_v=64, n_sink=3, window=10, scale=0.1):
        return B.lib().loza_ssa_decode_f32(q, FAKE, vc, lens, FAKE, FAKE, 2, Hq, Hkv, S, d_qk, d_v, n_sink, window, scale, None)
    assert call(q=None) == ERR_NULL and call(lens=None) == ERR_NULL
    assert call(vc=FAKE, d_v=96) == ERR_SHAPE            # aliased values wider than the keys
    assert call(window=0) == ERR_SHAPE and call(Hq=3) == ERR_SHAPE and call(S=0) == ERR_SHAPE
    assert call(d_qk=257) == ERR_UNSUPPORTED
    assert call(q=FAKE + 4) == ERR_ALIGN and call(lens=FAKE + 2) == ERR_ALIGN
    assert B.lib().loza_ssa_decode_blocks_f32(FAKE, FAKE, FAKE + 64, FAKE, FAKE, FAKE, 2, 4, 2, 100, 64, 64,
                                              1, 0, 16, 0.1, None) == ERR_SHAPE


def test_alpha_gradient_rejects_bad_arguments_and_sizes_its_workspace():
    call = lambda d=FAKE, dalpha=FAKE, n=4096, ws=FAKE, wsb=1 << 20: B.lib().loza_ssa_calibration_alpha_grad(
        d, FAKE, FAKE, dalpha, n, ws, wsb, None)
    assert call(d=None) == ERR_NULL and call(dalpha=None) == ERR_NULL
    assert call(n=0) == ERR_SHAPE and call(n=12) == ERR_SHAPE
    assert call(ws=None) == ERR_WORKSPACE and call(wsb=8) == ERR_WORKSPACE
    assert call(d=FAKE + 8) == ERR_ALIGN and call(dalpha=FAKE + 2) == ERR_ALIGN
    assert B.loza_ssa_calibration_alpha_grad_workspace_bytes(12) == 0
    assert B.loza_ssa_calibration_alpha_grad_workspace_bytes(8) == 8                  # one workgroup, one double
    assert B.loza_ssa_calibration_alpha_grad_workspace_bytes(1 << 33) == 4096 * 8     # never more than 4096 partial sums


def test_the_header_is_plain_c_and_the_library_links_from_c(tmp_path):
    """gcc -std=c99 -pedantic -Werror on a program that includes the header, links the library and calls
    the host-only entry points; its output must agree with the Python binding's."""
    import shutil
    import subprocess
    from pathlib import Path
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    root = Path(__file__).resolve().parents[1]
    lib_dir = Path(B.LIB_PATH).parent
    exe = tmp_path / "abi_host"
    subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", str(root / "include"),
                    str(root / "tests" / "c" / "abi_host.c"), "-o", str(exe), "-L", str(lib_dir), "-lloza_ssa",
                    f"-Wl,-rpath,{lib_dir}", "-Wl,-rpath,/opt/rocm/lib"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.splitlines()
    got = {line.split()[0]: line.split()[1:] for line in out}
    assert got["live_ranges"] == ["0"] + [str(x) for x in B.loza_ssa_live_ranges(10000, 128, 512)]
    assert got["live_ranges_blocks"] == ["0"] + [str(x) for x in B.loza_ssa_live_ranges_blocks(1000, 1, 7, 128)]
    assert got["live_pairs"] == [str(B.loza_ssa_live_pairs(131072, 128, 8192))]
    assert got["live_pairs_blocks"] == [str(B.loza_ssa_live_pairs_blocks(131072, 1, 7, 128))]
    assert got["decode_splits"] == [str(B.loza_ssa_decode_num_splits(64, 64, 1, 262144, 128, 8192))]
    assert got["decode_ws"] == [str(B.loza_ssa_decode_workspace_bytes(64, 64, 1, 262144, 512, 128, 8192))]
    assert got["backward_ws"] == [str(B.loza_ssa_backward_workspace_bytes(1, 64, 1, 131072, 576, 512, 128, 8192, True))]
    assert got["calibration_ws"] == [str(B.loza_ssa_calibration_workspace_bytes(1, 64, 4096, 512))]
    assert got["alpha_grad_ws"] == [str(B.loza_ssa_calibration_alpha_grad_workspace_bytes(4096))]
    assert got["null_q"] == [str(ERR_NULL)]
    assert " ".join(got["status"]) == B.loza_status_str(ERR_WORKSPACE)


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", tmp_path / "nope.so")
    with pytest.raises(FileNotFoundError):
        B.lib()
