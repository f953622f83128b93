"""LOMO fused backward + update hot path for AMD MI355X: thin Python binding over liblomo.so.

The arithmetic lives in hand-written HIP kernels behind the C ABI declared in include/lomo.h;
this package only marshals arguments (torch tensors -> device pointers, sizes, stream).
There is no CPU fallback: without the built library every call raises.
"""
from .binding import (LomoError, library_path, load_library, lomo_version, lomo_status_str, lomo_wgrad_sqnorm,
                      lomo_embedding_sqnorm, lomo_vector_sqnorm, lomo_clip_coef, lomo_scaler_step,
                      lomo_reduce_flags, lomo_linear_backward_update, lomo_embedding_update,
                      lomo_vector_update, lomo_embedding_workspace_bytes, lomo_vector_workspace_bytes,
                      lomo_embedding_grouping, lomo_timing_enable, lomo_timing_read, KERNEL_FAMILIES,
                      lomo_step_workspace_bytes, lomo_step_norm_pass, lomo_step_update_pass, make_tensor_list,
                      lomo_linear_backward_update_clip_value, lomo_step_update_pass_clip_value,
                      lomo_wgrad_sqnorm_route, lomo_step_workspace_min_bytes, NORM_ALGORITHMS, LomoTensor, LomoStepOptions,
                      lomo_step_scalars_device, lomo_step_update_pass_device, unpack_step_scalars, SCALARS_BYTES,
                      lomo_linear_dgrad, lomo_swiglu_backward, lomo_rmsnorm_backward, lomo_attention_backward,
                      lomo_linear_forward, lomo_rmsnorm_forward, lomo_swiglu_forward, lomo_rope_forward,
                      lomo_attention_forward, lomo_cross_entropy, lomo_embedding_forward, lomo_linear_forward_residual,
                      lomo_cross_entropy_mean, lomo_vector_update_static, VECTOR_STATIC_BYTES, lomo_probe_mfma, lomo_probe_copy, PROBE_OPERAND_BYTES, on_stream,
                      EXPORTED_SYMBOLS)

__all__ = [n for n in dir() if n.startswith("lomo_")] + ["LomoError", "library_path", "load_library",
                                                         "EXPORTED_SYMBOLS"]
