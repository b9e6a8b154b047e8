"""MI355X-native HyperAttention forward pass (arXiv 2310.05869).

The computation lives in libhyperattn.so (hand-written HIP for gfx950, C ABI
declared in include/hyperattn.h); this package is its thin Python binding.
"""
from .binding import (  # noqa: F401
    HA_BF16, HA_FP32, HaAlg2Options, HaAlg2WsLayout, HaBwdWsLayout, HaParams, HaShape, HaWsLayout, HyperAttnError, alg2_workspace_views, alloc_backward_workspace, alloc_workspace, exact_attn_backward, exact_attn_forward,
    exported_symbols, ha_block_attn, ha_gather_rows, ha_lsh_hash, ha_alg2_workspace_layout, ha_backward_workspace_bytes, ha_make_projection, ha_make_samples, ha_issue_probe_count, ha_measure_hbm_rate, ha_measure_issue_rates, ha_measure_mfma_rate,
    ha_merge_unpermute, ha_sampled_attn, ha_seg_sort, ha_workspace_bytes, ha_workspace_layout, hyperattn_backward, hyperattn_backward_timed, hyperattn_forward, hyperattn_forward_alg2, hyperattn_forward_static, hyperattn_forward_timed, ha_static_scratch_bytes, ha_forward_workgroups, hyperattn_forward_stamped, STAMP_NAMES, STAMP_WORDS, stamp_place,
    lib, make_params, make_shape, strerror, workspace_views,
)
