"""MI355X-native quantized linear layers (the deployment hot path of MixDQ, arxiv 2405.17873).

Thin Python binding over the C ABI declared in include/mixdq.h.  Every step of the path runs in the
HIP kernels of libmixdq.so; this package only marshals arguments.  There is no CPU fallback.
"""
from .binding import (  # noqa: F401
    BF16, F16, a8_row_bytes, builtin_workspace_bytes, qlinear_a8_builtin_ws, alloc_search, alloc_solve, alloc_split_budget, conv3x3_a8, conv3x3_a8_workspace_bytes, conv3x3_w_only, conv_tap_sums, plan_qlinear_a8_codes, plan_qlinear_a8_geglu, plan_qlinear_a8_geglu_dynamic, qlinear_w_only_geglu, qlinear_a8_codes, qlinear_a8_geglu, qlinear_a8_geglu_dynamic, qlinear_a8_geglu_dynamic_workspace_bytes, qlinear_w_only_geglu, qlinear_w_only_geglu_a8, LAYOUT_CANONICAL, LAYOUT_KERNEL, MixdqError, PackedWeight, bos_aware_kv_proj, keep_weights_16bit,
    bos_aware_kv_proj_workspace_bytes, lib_path, load, pack_weights, packed_bytes, plan_bos_aware_kv_proj, plan_qlinear_a8, plan_qlinear_w_only, prof_bracket_overhead_us, prof_copy, prof_microbench, machine_peaks, prof_enable, prof_filter, prof_phase_buffer, prof_read, prof_reset, qlinear_a8_workspace_bytes,
    qlinear_w2a8, qlinear_w4a8, qlinear_w8a8, qlinear_w_only, quantize_weights, split_workspace_bytes, stack_weights, tune_force_band, tune_force_splits, tune_force_tile, unpack_weights, version)
