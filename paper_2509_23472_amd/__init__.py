"""LoRAct activation compression for AMD MI355X: Python binding of the libloract C ABI."""
from .api import (BF16, F32, MAX_RANK, STATUS_RANK_DEFICIENT, LoractError, loract_compress,
                  loract_compress_adaptive,
                  loract_gaussian_omega_t, loract_lora_grad, loract_lora_grad_static,
                  loract_static_scratch_bytes, loract_prenorm_backward,
                  loract_prenorm_forward, loract_profile_begin,
                  loract_profile_end, loract_reconstruct, loract_rsvd, loract_sample_indices,
                  loract_version, loract_workspace_bytes, make_params)

__all__ = [
    "BF16", "F32", "MAX_RANK", "STATUS_RANK_DEFICIENT", "LoractError", "loract_compress", "loract_compress_adaptive",
    "loract_gaussian_omega_t", "loract_lora_grad", "loract_lora_grad_static",
    "loract_static_scratch_bytes", "loract_prenorm_backward", "loract_prenorm_forward",
    "loract_profile_begin", "loract_profile_end",
    "loract_reconstruct", "loract_rsvd", "loract_sample_indices", "loract_version",
    "loract_workspace_bytes", "make_params",
]
