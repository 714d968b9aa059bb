"""MI355X-native time-to-first-token path of KV Prediction (arXiv 2410.08391).

The product is `libkvp.so` (hand-written HIP for gfx950 behind a C ABI, see
`include/kvp.h`).  This package is a thin ctypes binding with the same names;
PyTorch is used only for device memory and streams.  Importing the package
does not load the library; the first call that needs it does, and fails loudly
if it has not been built (`python -m paper_2410_08391_amd.build`).
"""
from .binding import (KVP, KVPError, lib, library_path, kvp_load_weights, kvp_workspace_bytes,  # noqa: F401
                      kvp_prefill_predict, kvp_run_stages, kvp_free, kvp_last_error, kvp_version,
                      kvp_reference_workspace_bytes, kvp_reference_prefill, MODEL_BASE, MODEL_AUX,
                      kvp_generation_workspace_bytes, kvp_generation_step, kvp_generation_step_static,
                      kvp_static_scratch_bytes, kvp_check_flags, kvp_debug_plan, kvp_probe_mfma, kvp_probe_stream, kvp_debug_flash_guard, FLAG_TOKEN_CLAMPED, EXPORTS,
                      STAGE_AUX, STAGE_PREDICT, STAGE_BASE, STAGE_ALL, STAGE_BASE_ABSORBED, KERNEL_CLASSES)
