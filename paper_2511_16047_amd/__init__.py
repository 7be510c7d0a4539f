"""AMS-KV hot path for AMD MI355X: HIP kernels behind a C ABI (include/amskv.h) and a thin
ctypes binding with the same call names."""
from .binding import *  # noqa: F401,F403
from .binding import AmskvError, load_library, status_string  # noqa: F401
