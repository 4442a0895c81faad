"""AirCache hot path for MI355X: hand-written HIP (gfx950) behind a C ABI, with a ctypes binding."""
from .binding import (  # noqa: F401
    AIR_BF16,
    AIR_BUDGET_SKEW,
    AIR_BUDGET_STRENGTH,
    AIR_BUDGET_STRENGTH_SKEW,
    AIR_BUDGET_UNIFORM,
    AIR_F32,
    AIR_WINDOW_TEXT,
    AIR_WINDOW_VISUAL,
    AirCache,
    AirError,
    air_config,
    air_layer,
    air_seq,
    air_strides,
    load_library,
    make_config,
)
