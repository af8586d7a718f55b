"""MI355X-native training step (forward, pullbacks, SGD-momentum) behind a C ABI.

`binding` mirrors include/s4tf.h one to one; `build` compiles libs4tf.so for gfx950."""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
