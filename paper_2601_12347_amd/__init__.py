"""MI355X-native incremental GNN inference on evolving graphs (hot path of
RIPPLE++): HIP kernels behind a C ABI (include/ripple.h) plus this thin
ctypes binding. Nothing is loaded at import time; the first call dlopens
libripple.so and fails loudly if it is missing."""
from .binding import *          # noqa: F401,F403
from .binding import (LIB_PATH, EXPORTS, RippleError, load_library, BatchResult, Stats, PHASES,
                      OPT_TIMING, OPT_SCATTER_MODE, OPT_PULL_RATIO, OPT_PROJECT_FIRST, OPT_BF16_MFMA, OPT_SELF_CACHE, OPT_DETERMINISTIC, OPT_SPLIT_MFMA, OPT_SPARSE_FRONTIER,
                      OPT_ROW_SEGMENTS, OPT_PACKED_MESSAGES, OPT_STREAM_TRANSFORM, OPT_SORTED_MESSAGES)
