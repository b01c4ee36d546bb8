"""Low-rank binary index (arXiv 1905.05686) inference path for MI355X.

Thin Python binding over the C ABI in include/lrbi.h (argument marshalling
only).  Every step of the method runs in the HIP kernels of liblrbi.so; there
is no CPU or PyTorch fallback: if the library is missing, calls raise.
"""
from .binding import (  # noqa: F401
    BF16, F16, F32, STATIC_SCRATCH_BYTES, FLAG_DECODE_GENERIC, FLAG_PATH_MFMA, FLAG_PATH_STREAM, FLAG_PATH_VALU, Desc, LrbiError, csr_bits, decode_and_gemm, decode_mask,
    flag_splitk, flag_tile, index_bits, index_bits_ranked, library_path, load_library, lstm_step,
    lstm_step_workspace_bytes, masked_conv3x3, masked_conv3x3_workspace_bytes, masked_gemm, masked_gemm_t,
    masked_gemm_t_workspace_bytes, masked_gemm_static, masked_gemm_workspace_bytes, masked_grad, nmf, nmf_workspace_bytes,
    pack_factors, search_thresholds, search_workspace_bytes, strerror, threshold_eval, threshold_eval_workspace_bytes,
    unpack_mask,
)
