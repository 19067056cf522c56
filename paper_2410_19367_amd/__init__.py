"""MI355X-native stage compute for the BitPipe schedule: thin binding over libbitpipe_stage.so."""
from .binding import *  # noqa: F401,F403
from . import binding  # noqa: F401
