"""MI355X-native AdaptGear aggregation path (arXiv 2305.17408).

The product is libadaptgear.so (HIP kernels + C ABI, see include/adaptgear.h);
this package is its thin Python binding.
"""
from .binding import *  # noqa: F401,F403
from .binding import lib, LIB_PATH, EXPORTS, AdaptGearError  # noqa: F401
