"""XCD-aware swizzled bf16 GEMM for AMD Instinct MI355X: thin Python binding over libswz.

Every step of the path (PID remap, raster decode, staging, MFMA loop, epilogue) runs inside
the library's HIP kernels; this package only marshals arguments.  Importing it loads
``libswz.so`` and fails loudly if the library has not been built (there is no fallback).
"""
from .binding import (  # noqa: F401
    MODE_GROUPM, MODE_RR, MODE_SKEW, MODE_XCD, MODE_XCD_GROUPM, MODES, DTYPE_BF16, SwzError, SwzParams, copy_bytes, device_info, gemm,
    gemm_plan, lib, pid_map, pid_map_device, pid_map_persistent, pid_map_persistent_device, status_string, transpose,
    layernorm, mfma_peak, softmax, gemm_probe, PROBE_WORDS,
)
