"""MI355X-native co-located inference on pooled CU-masked streams (libeclip + ctypes binding)."""
from .binding import *  # noqa: F401,F403
