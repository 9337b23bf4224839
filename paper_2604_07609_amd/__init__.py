"""Python binding of libblink (the on-GPU serving step of Blink for MI355X).

Argument marshalling only: every step of the serving path runs in the HIP library. The
library must have been built (python -m paper_2604_07609_amd.build); importing fails
loudly otherwise. There is no CPU fallback.
"""
from .binding import (Engine, BlinkError, sample_rows, sample_rows_static, lib_path, load_library, EXPORTS, FLAG_TRACE, FLAG_EXIT_WHEN_IDLE,  # noqa: F401
                      FLAG_KEEP_LOGITS, FLAG_NO_GRAPH, FLAG_CHUNKED_PREFILL, FLAG_PREEMPTION, FLAG_PREFIX_CACHE, FLAG_SPECULATIVE, FLAG_HOST_STEP, ERR_INVAL, ERR_TOO_LARGE, ERR_FULL, ERR_DEVICE, ERR_STATE,
                      EVENT_FIRST, EVENT_LAST, DBG)
