"""MI355X-native hot path of Reward-Guided Speculative Decoding: ctypes binding
over ``librsd.so`` (hand-written HIP kernels behind the C ABI of
``include/rsd.h``).  There is no CPU fallback: importing :mod:`.binding`
without the built library raises."""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
