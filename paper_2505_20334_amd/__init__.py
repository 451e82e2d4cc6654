"""MI355X-native hot path of Lookahead Q-Cache (LAQ) re-eviction (paper Sec. 4.3, Eq. 4).

The work is done by hand-written HIP kernels behind the C ABI declared in
``include/laq.h``; this package only marshals arguments (``binding``) and knows how
to compile the library (``_build``).  There is no CPU fallback: if the shared
library is missing the first call builds it with hipcc, and raises if that fails.
"""
from .binding import (LaqError, laq_compact, laq_init, laq_workspace_status, laq_score_kernel, laq_decode_attention, laq_decode_workspace_bytes, laq_evict, laq_qcache_store, laq_recall, laq_score, laq_select,  # noqa: F401
                      laq_select_sink_recent, laq_strerror, laq_workspace_bytes, lib_path, load_library, packed_rows)

__all__ = ["LaqError", "laq_compact", "laq_init", "laq_workspace_status", "laq_score_kernel", "laq_decode_attention", "laq_decode_workspace_bytes", "laq_evict", "laq_qcache_store", "laq_recall", "laq_score", "laq_select", "laq_select_sink_recent", "laq_strerror",
           "laq_workspace_bytes", "lib_path", "load_library", "packed_rows"]
