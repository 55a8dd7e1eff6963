"""MI355X-native spherical attention (neighborhood and global), C ABI + thin binding."""
from .binding import *  # noqa: F401,F403
