"""MI355X-native per-example clipped-gradient step of DP-SGD (clip, accumulate, noise, Adam with
decoupled weight decay) behind the C ABI of include/dpclip.h.  The library is loaded on first use."""
from .binding import *  # noqa: F401,F403
from .binding import Context, DpError, load_library  # noqa: F401
from .step import StepRunner  # noqa: F401,E402
