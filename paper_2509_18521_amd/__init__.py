"""MI355X-native APRIL rollout engine: ctypes binding over libapril.so (HIP, gfx950)."""
from .binding import *  # noqa: F401,F403
from .binding import load_library, make_cfg, pack_weights  # noqa: F401
