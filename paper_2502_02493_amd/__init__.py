"""MI355X-native EasySpec draft hot path: layer-parallel fuzzy draft step, bonus calibration
and greedy acceptance behind a C ABI (include/easyspec.h), bound here with ctypes."""
from .binding import *  # noqa: F401,F403
from .binding import (EXPORTS, LIB_PATH, EasySpecError, easyspec_config, load_library, make_config)
