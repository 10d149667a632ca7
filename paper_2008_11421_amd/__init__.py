"""MI355X-native out-of-core training step (KARMA, SC20): thin Python binding over
libkarma.so.  All computation happens in the library's HIP kernels and host runtime."""
from .binding import *  # noqa: F401,F403
