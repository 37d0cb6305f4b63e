"""MI355X-native GPU side of hybrid CPU/GPU A3C (arXiv 1611.06256).

Thin Python binding over the C ABI in ``include/ga3c.h``; every step of the
path runs in the HIP library, this package only marshals arguments.
"""
from .binding import (  # noqa: F401
    Ga3c, Ga3cError, HParams, NetDesc, TrainStats, SMALL_NET, LARGE_NET, Scheduler, Tuner, lib_path, load_library,
    rmsprop_flat, predict_static, STATIC_MAX_FRAMES,
)
