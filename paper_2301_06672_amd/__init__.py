"""MI355X-native IVFPQ search (arXiv 2301.06672): thin Python binding over libivfpq.so."""
from .binding import (  # noqa: F401
    Index, IvfpqError, lib, EXPORTS, LIB_PATH, ivfpq_assign_device, ivfpq_refine, ivfpq_stream_read,
    LUT_FP32, LUT_FP16, LUT_FP8_E5M3, LUT_FP8_E4M4, LUT_NAMES, LUT_BYTES, MAX_K, MAX_PROBES,
    ROUND_NEAREST, ROUND_TRUNCATE, STATIC_SCRATCH_BYTES,
    TUNE_SCAN_THREADS, TUNE_ORDER_BLOCK, TUNE_SCAN_SHARE, TUNE_EARLY_EXIT, TUNE_LDS_PAD,
    OK, EINVAL, ENOSPACE, EHIP, EUNSUPPORTED, ESTATE,
)
