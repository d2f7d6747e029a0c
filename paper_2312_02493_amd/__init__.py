"""MI355X-native AR-Topk gradient compressor (one GPU, W simulated workers).

The compute lives in libartopk.so (hand-written HIP for gfx950) behind the C
ABI of include/artopk.h; this package only marshals arguments.  There is no CPU
fallback: using the library without the built extension raises.
"""

from .binding import (  # noqa: F401
    ARTOPK_OPT_GUESS_MIN_N, ARTOPK_OPT_LEADER_FIRST, ARTOPK_OPT_NONTEMPORAL, ARTOPK_OPT_STAGE_TILES,
    ARTOPK_OPT_UPDATE_TILES_MIN_N,
    artopk_scratch_bytes, artopk_variance_static,
    ARTOPK_FIXED, ARTOPK_G_BF16, ARTOPK_G_F16, ARTOPK_G_F32, ARTOPK_STAR, ARTOPK_STAR_COUNTER, ARTOPK_VAR, ARTOPK_VAR_G, ARTOPK_VAR_TOPK, ArTopkError, Context,
    exported_symbols, lib_path, load_library,
)
