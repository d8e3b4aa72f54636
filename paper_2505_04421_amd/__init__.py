"""MI355X-native LONGER forward / KV-cache serving path.

Thin ctypes binding over ``liblonger.so`` (C ABI in ``include/longer.h``): the
functions here carry the same names as the C entry points and only marshal
arguments -- every step of the path runs in the library's HIP kernels.  PyTorch
is used for device memory and streams only.  There is no CPU fallback: if the
library is missing, or no GPU is present when a compute call is made, the call
raises.
"""
from .binding import (  # noqa: F401
    LongerError, DeviceModel, load_library, library_path, make_config, exported_symbols,
    longer_workspace_bytes, longer_kv_cache_bytes, longer_inner_transformer, longer_token_merge,
    longer_hybrid_cross_attn, longer_self_attn_layer, longer_forward, longer_kv_cache_build,
    longer_score_candidates, longer_input_generation, longer_forward_from_inputs, longer_kv_cache_build_from_inputs, CInputWeights, longer_probe_mfma_layout, longer_last_error,
    longer_stage_timing, longer_stage_timing_read, STAGES,
    longer_packed_weights_bytes, longer_pack_weights, longer_score_candidates_static, longer_probe_rate, CWeights,
    longer_backward_workspace_bytes, longer_block_grad_floats, longer_token_merge_backward, block_grad_views,
    longer_model_grad_floats, longer_forward_backward_workspace_bytes, longer_forward_backward, model_grad_views,
    longer_input_backward_workspace_bytes, longer_input_grad_floats, longer_input_generation_backward, input_grad_views,
)
