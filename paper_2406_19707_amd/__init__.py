"""MI355X-native InfiniGen rehearsal + sparse decode attention (thin binding over libinfinigen_hip)."""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
