"""MI355X-native BUZZ sparse-KV-cache decode path (arxiv 2410.23079): thin Python binding over ``libbuzz.so``."""
from .binding import (bench_copy, BuzzCache, BuzzConfig, BuzzError, FLAG_AUTO_EVICT, FLAG_CACHED, FLAG_DETERMINISTIC, FLAG_DEVICE_MERGE, FLAG_DRY_RUN, FLAG_GLOBAL_TOPK, FLAG_INTERVAL_NEW, FLAG_LOG_N, FLAG_STREAMING,
                      FLAG_THRESHOLD_TOTAL, library_path, suggest_threshold, load_library,
                      workspace_bytes)

__all__ = ["bench_copy", "BuzzCache", "BuzzConfig", "BuzzError", "FLAG_AUTO_EVICT", "FLAG_CACHED", "FLAG_DETERMINISTIC", "FLAG_DEVICE_MERGE", "FLAG_DRY_RUN", "FLAG_GLOBAL_TOPK", "FLAG_INTERVAL_NEW", "FLAG_LOG_N", "FLAG_STREAMING",
           "FLAG_THRESHOLD_TOTAL", "suggest_threshold", "library_path",
           "load_library", "workspace_bytes"]
