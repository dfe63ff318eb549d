"""MI355X-native forward pass of Generalized Depthwise-Separable convolutions (HIP kernels behind a C ABI)."""
from .binding import *          # noqa: F401,F403
from .binding import lib, LIB_PATH, EXPORTS, GdwsError, LayerDesc, Plan, Net, Graph, make_desc   # noqa: F401
