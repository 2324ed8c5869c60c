"""MI355X-native population-update path of WASH (arXiv 2405.17517):
wash_shuffle (Eq. 3), wash_average (Alg. 1 output), papa_ema (Eq. 1) as
hand-written gfx950 kernels behind a C ABI (include/wash.h)."""
from .binding import (  # noqa: F401
    MAX_N, OPT_AVERAGE_CHUNKS, OPT_DENSE, OPT_GAP_BLOCKS, OPT_SHUFFLE_BLOCKS_PER_CU, OPT_STREAM_MIN_BYTES, OPT_TILE_COORDS, SegmentList, WashError, papa_ema, wash_average, wash_consensus_sqdist, wash_consensus_sqdist_noalloc, wash_copy_f32, wash_probe_scattered, wash_weighted_average, wash_layer_probs,
    wash_set_option, wash_shuffle, wash_shuffle_gap, wash_shuffle_device_step, wash_shuffle_states, wash_shutdown,
)
from .placement import place_population  # noqa: F401,E402
