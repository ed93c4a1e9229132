"""The index set of the kernels, read back bit-exactly at the full benchmark shapes.

Probe: with Q = 0 every live key of a query gets the weight 1 / |live(i)| and the log-sum-exp is
ln |live(i)|; with a value tensor that is one-hot (V[j_c, c] = 1 for chosen probe keys j_c, one per
output column) the output column c of query i is non-zero exactly when key j_c is live for i. One
launch at the benchmark shape therefore reads back as many columns of the kernel's mask as the
value width, for every query row at once. The probe keys sit on every edge of the pattern for a set of
query rows (end of the sink, trailing edge of the window, the causal diagonal, key-tile and row-tile
boundaries next to them); those rows are compared with the oracle's explicit mask key by key, and
the log-sum-exp of EVERY row of the launch is compared with ln |live(i)| (|live(i)| in closed form;
tests/test_oracle_pins*.py hold the closed forms against the oracle's explicit masks).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_23966_amd import workloads as W
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _probe_rows(S, T, row_tile_positions):
    """Query positions whose masks are compared key by key."""
    rows = {0, 1, T - 2, T - 1, T, T + 1, S - 1, S - 2, S // 2, S // 2 + 1, S // 3}
    for t in (T // row_tile_positions + 1, S // (2 * row_tile_positions), S // row_tile_positions - 1):
        for d in (-1, 0, 1):
            rows.add(t * row_tile_positions + d)
    rng = np.random.default_rng(99)
    rows |= set(int(x) for x in rng.integers(T, S, size=6))
    return sorted(r for r in rows if 0 <= r < S)


def _probe_keys(rows, S, n_sink, win_begin_of, n_cols):
    """Up to n_cols probe keys: the pattern's edges for each probe row, nearest first."""
    keys = []
    def add(j):
        if 0 <= j < S and j not in keys and len(keys) < n_cols:
            keys.append(j)
    for d in (-2, -1, 0, 1):
        add(n_sink + d)
    for i in rows:
        wb = win_begin_of(i)
        for j in (wb - 1, wb, wb + 1, i - 1, i, i + 1, wb - 2, (wb // 32) * 32 - 1, (wb // 32) * 32, (wb // 32) * 32 + 32,
                  (i // 32) * 32, (i // 32) * 32 - 1, (i // 32) * 32 + 32):
            add(j)
    rng = np.random.default_rng(7)
    while len(keys) < n_cols:
        add(int(rng.integers(0, S)))
    return np.asarray(keys, dtype=np.int64)


def _run_probe(cfg, dev, pattern, block, rows, keys, live_mask_of, live_count_of):
    """One launch at cfg's shape with Q = 0 and one-hot values on `keys`; checks the listed rows
    against the oracle's mask and every row's log-sum-exp against ln |live(i)|."""
    S, Hq, d_v = cfg.S, cfg.Hq, cfg.d_v
    q = torch.zeros(cfg.B, S, Hq, cfg.d_qk, dtype=torch.bfloat16, device=dev)
    k = torch.zeros(cfg.B, S, cfg.Hkv, cfg.d_qk, dtype=torch.bfloat16, device=dev)
    cols = torch.arange(len(keys), device=dev)
    v = k if cfg.alias_v else torch.zeros(cfg.B, S, cfg.Hkv, d_v, dtype=torch.bfloat16, device=dev)
    for g in range(cfg.Hkv):
        v[0, torch.as_tensor(keys, device=dev), g, cols] = 1.0
    out, lse = H.run_prefill(q, k, v, pattern[0], pattern[1], 1.0, d_v=d_v, block=block)
    # every row, every head: lse = ln |live(i)|
    i_all = np.arange(S, dtype=np.int64)
    want_lse = torch.as_tensor(np.log(live_count_of(i_all).astype(np.float64)), device=dev)
    err = (lse[0].double() - want_lse[None, :]).abs().max().item()
    print(f"[probe] {cfg.name} b{block}: max |lse - ln|live|| over all {S * Hq} rows = {err:.2e}", flush=True)
    assert err <= 1e-5, f"log-sum-exp of a row does not match its live count (max error {err})"
    # the probe rows: out != 0 exactly on the live probe keys, for the first and the last head of a group
    want = np.stack([live_mask_of(i)[keys].astype(bool) for i in rows])
    for h in sorted({0, Hq - 1, Hq // 2}):
        vals = out[0, torch.as_tensor(rows, device=dev), h, : len(keys)].float().cpu().numpy()
        got = vals != 0
        for r, i in enumerate(rows):
            assert (got[r] == want[r]).all(), (f"{cfg.name}: query {i} head {h}: kernel and oracle disagree on keys "
                                               f"{keys[got[r] != want[r]][:8]}")
            # the weights are 1 / |live(i)| where live
            np.testing.assert_allclose(vals[r][want[r]], 1.0 / live_count_of(np.int64(i)), rtol=2.0 ** -8)
    del q, k, v, out, lse
    torch.cuda.empty_cache()


def _token_case(cfg, dev):
    S, ns, win = cfg.S, cfg.n_sink, cfg.window
    T = ns + win
    rows = _probe_rows(S, T, max(1, 128 * cfg.Hkv // cfg.Hq))
    keys = _probe_keys(rows, S, ns, lambda i: max(0, i - win + 1), cfg.d_v)
    _run_probe(cfg, dev, (ns, win), None, rows, keys,
               lambda i: oracle.live_mask(i, S, ns, win), lambda i: H.live_count_tokens(i, ns, win))


def test_index_set_cfg2_shape(gpu_device):
    _token_case(W.CFG2, gpu_device)


def test_index_set_cfg3_shape(gpu_device):
    _token_case(W.CFG3, gpu_device)


def test_index_set_cfg5_shape(gpu_device):
    free, _ = torch.cuda.mem_get_info()
    if free < 160 * 2 ** 30:
        pytest.skip("the 1M-token configuration needs 150 GB of free HBM")
    _token_case(W.CFG5, gpu_device)


def test_index_set_paper_block_pattern_128k(gpu_device):
    """(s, l, b) = (1, 7, 128) of the paper's Training section, at the 128K MLA shape."""
    cfg = W.CFG3
    S, s, l, b = cfg.S, 1, 7, 128
    rows = _probe_rows(S, (s + l) * b, 2)
    rows = sorted(set(rows) | {b * 9 - 1, b * 9, b * 500 + 127, b * 500 + 128})
    keys = _probe_keys(rows, S, s * b, lambda i: max(0, i // b - l + 1) * b, cfg.d_v)
    _run_probe(cfg, gpu_device, (s, l), b, rows, keys,
               lambda i: oracle.live_mask_blocks(i, S, s, l, b), lambda i: H.live_count_blocks(i, s, l, b))
