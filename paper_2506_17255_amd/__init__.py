"""MI355X-native fused sketch-query linear layer (UltraSketchLLM inference
hot path).  The package is a thin binding over libsketch_linear.so."""
from .binding import *  # noqa: F401,F403
from .binding import (EXPORTS, SketchLinearError, load_library, make_desc, skl_desc_t, skl_info_t)  # noqa: F401
