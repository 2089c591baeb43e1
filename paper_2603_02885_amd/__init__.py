"""MI355X-native multiplexed multi-task PEFT linear layer (C-ABI library + thin binding)."""
from .binding import *  # noqa: F401,F403
