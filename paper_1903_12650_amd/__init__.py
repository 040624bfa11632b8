"""MI355X-native ResNet-50 large-minibatch training step (hand-written HIP kernels
behind a C ABI; see include/rn50_hip.h).  This package is the thin Python binding:
argument marshalling only, every computation runs in the library's kernels."""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
