"""MI355X-native SRM generation: thin Python binding over libsrm (include/srm.h).

Every step of the path runs in the HIP library; this package only marshals
arguments.  PyTorch is used for device memory and streams.  There is no CPU
fallback: if the library is missing, loading fails.
"""
from .binding import (SRM_BF16, SRM_FP32, Model, SrmError, lib, linear, linear_argmax_noalloc, linear_timeline_probe,
                      linear_argmax_noalloc_max_bytes, linear_scratch_bytes,
                      prefill_ragged_plan, probe_copy, probe_mfma, sample_logits,
                      workspace_bytes_config)  # noqa: F401
