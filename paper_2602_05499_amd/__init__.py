"""MI355X-native speculative draft-and-verify decode step (SDFP hot path): Python binding of libsdfp.

Argument marshalling only -- every step of the path runs in the HIP kernels behind the C-ABI declared in
include/sdfp.h.  PyTorch is used for device memory and streams, nothing else.  There is no CPU fallback:
if the built library is missing, loading fails.
"""
from .binding import (  # noqa: F401
    SD_F32, SD_BF16, SD_GREEDY, SD_SAMPLE, SD_LOGITS_DRAFT, SD_LOGITS_VERIFY, SD_OK, SD_EINVAL, SD_ECAPACITY,
    SD_ESTATE, SD_EHIP, SD_ENOMEM, SD_ETIMEOUT, SD_MAX_K, SD_STATIC_WS_BYTES, SD_STATIC_MAX_LAYERS, SdConfig, SdWeights, SdStats, SdError, load_library, library_path,
    sd_kv_bytes, sd_workspace_bytes, sd_init, sd_init_static, sd_set_skip_mask, sd_prefill, sd_draft, sd_verify, sd_accept,
    sd_rollback, sd_decode, sd_set_pending, sd_set_draft, sd_read, sd_dump_logits, sd_dump_draft, sd_keep_logits,
    sd_phase_trace, sd_phase_trace_read, sd_set_prefill_mode, sd_sync, sd_last_hip_error, sd_free, sd_strerror, EXPORTED_SYMBOLS,
)
from .session import Session, build_library  # noqa: F401
