"""MI355X-native selective-KV-recompute prefill (hot path of KEEP, arxiv 2602.23592).

The compute lives in libkeep_hip.so (HIP kernels for gfx950 behind the C ABI of
include/keep.h and include/keep_memory.h); `binding` marshals torch tensors into it.
"""
from . import binding  # noqa: F401
from .binding import (KeepContext, KeepMemory, KeepPrompt, KeepError, load_library)  # noqa: F401
