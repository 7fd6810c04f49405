"""MI355X-native NVFP4 linear layer of Quartet II (quantizers RTN / SR / MS-EDEN and the
block-scaled GEMMs) behind the C ABI of include/qii.h.  See binding.py for the calls."""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
