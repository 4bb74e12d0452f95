"""MI355X-native direct sparse convolution (Escoin): C-ABI HIP library plus a thin binding."""
from . import workloads  # noqa: F401
from .binding import *  # noqa: F401,F403
from .binding import (EscoinError, F_BIAS, F_RELU, desc_of, escoin_conv_desc, lib,  # noqa: F401
                      make_desc, make_tuning, plan_header)
