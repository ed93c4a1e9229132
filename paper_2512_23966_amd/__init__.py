"""MI355X-native streaming sparse attention (the SSA hot path of LongCat ZigZag Attention).

The product is ``libloza_ssa.so`` (hand-written HIP for gfx950 behind the C ABI of
``include/loza_ssa.h``); this package is its Python binding plus the synthetic workload recipes.
"""
from .binding import (  # noqa: F401
    LIB_PATH, LOZA_OK, LOZA_WINDOW_INF, EXPORTS, LozaError, lib,
    loza_ssa_prefill, loza_ssa_prefill_f32, loza_ssa_decode,
    loza_ssa_decode_workspace_bytes, loza_ssa_decode_num_splits,
    loza_ssa_live_ranges, loza_ssa_live_pairs, loza_status_str,
    loza_ssa_prefill_blocks, loza_ssa_prefill_blocks_f32, loza_ssa_decode_blocks,
    loza_ssa_live_ranges_blocks, loza_ssa_live_pairs_blocks,
    loza_ssa_decode_paged, loza_ssa_decode_paged_blocks,
    loza_ssa_prefill_calibration_blocks, loza_ssa_calibration_workspace_bytes,
    loza_ssa_extend, loza_ssa_extend_blocks, loza_ssa_extend_paged, loza_ssa_extend_paged_blocks,
    loza_ssa_backward, loza_ssa_backward_blocks,
    loza_ssa_backward_workspace_bytes, loza_ssa_backward_workspace_bytes_blocks,
    loza_ssa_backward_f32, loza_ssa_backward_blocks_f32,
    loza_ssa_decode_f32, loza_ssa_decode_blocks_f32,
    loza_ssa_calibration_alpha_grad, loza_ssa_calibration_alpha_grad_workspace_bytes,
    loza_ssa_decode_static, LOZA_DECODE_STATIC_BYTES,
)
