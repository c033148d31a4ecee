"""MI355X-native LoRDS inference path: thin Python binding over liblords.so.

The package holds the HIP kernels (csrc/), the build script and this ctypes
binding.  Every step of the path runs in the kernels; Python only marshals
arguments.  There is no CPU fallback: if the library is missing the calls fail.
"""
from .binding import (  # noqa: F401
    LordsError, LORDS_BF16, LORDS_F32, LORDS_PATH_AUTO, LORDS_PATH_DECODE, LORDS_PATH_PREFILL, LORDS_PATH_MFMA,
    LORDS_PATH_GEMV, LORDS_PATH_SMALLM,
    STATUS_NAMES, library, library_path, lords_version, lords_status_string, lords_row_bytes,
    lords_equivalent_rank, lords_mixed_schedule, lords_unpack, bf16_from_bits, lords_dequant, lords_matmul,
    lords_matmul_ex, lords_matmul_ws, lords_matmul_noalloc, lords_workspace_bytes, lords_workspace_zero_bytes,
    lords_noalloc_limit, lords_probe_stream_read, lords_probe_mfma_bf16, lords_repack_bytes, lords_repack, lords_matmul_repacked,
    lords_quantize, lords_block_init, lords_matmul_batched, lords_gate_up,
    lords_transpose_codes, lords_backward_input, lords_backward_factors,
)
