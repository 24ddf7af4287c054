"""MI355X-native hot path of DISCO speculative decoding: ctypes binding over libdisco.so.

The binding marshals arguments only; every step of the path runs in the library's HIP kernels.
PyTorch is used for device memory and streams."""
from .binding import *  # noqa: F401,F403
