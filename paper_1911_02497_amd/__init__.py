"""Compression step of Condensa's L-C optimizer on MI355X: thin binding over libcondensa.so.

All arithmetic runs in the HIP kernels of the C-ABI library declared in include/condensa.h; this
package only marshals torch device tensors into pointers.  The library is loaded on first use and
loading fails loudly when it has not been built (``python -m paper_1911_02497_amd.build``).
"""
from .binding import (  # noqa: F401
    SCOPE_GLOBAL, SCOPE_PER_TENSOR, OPT_SELECT_PATH, OPT_SAMPLE_LOG2, OPT_WINDOW_MARGIN, OPT_CAND_SHIFT, OPT_PROFILE, OPT_APPLY_THREADS, OPT_FUSED_SWEEP, WINDOW_MARGIN_DEFAULT,
    CondensaError, Config, condensa_config, library, exported_symbols, TensorTable, tensor_table, condensa_prune, condensa_filter_prune, condensa_block_prune, condensa_block_prune_nd, condensa_neuron_prune, condensa_structure_prune,
    condensa_quantize, condensa_dequantize, condensa_quantize_bf16, condensa_dequantize_bf16, condensa_quantize_fp8, condensa_dequantize_fp8, FP8_E4M3, FP8_E5M2, condensa_lc_step, condensa_lc_step_pq, condensa_count_nonzero, condensa_thin, condensa_lc_sgd_step, condensa_mu_schedule, condensa_set_option, condensa_get_option,
    condensa_workspace_bytes, select_records, condensa_profile_read, condensa_profile_reset, condensa_launch_count,
)
