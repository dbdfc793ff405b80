"""MI355X-native ring-step attention (the per-device hot path of Double-Ring-Attention).

`binding` mirrors the C ABI of libloong.so one to one; `ring` replays one rank's
micro-steps on a single GPU.  Importing the package loads the HIP library and fails if it
has not been built (python -m paper_2406_18485_amd.build).
"""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
