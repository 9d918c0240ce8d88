"""MI355X-native hot path of OmniBal-style balanced VLM training: packed variable-length
transformer-block forward/backward (hand-written gfx950 kernels behind a C ABI) and the host-side
balanced mini-batch packer.  This package only marshals arguments; all arithmetic runs in
libomnibal.so.  There is no CPU fallback: importing `binding` without the built library raises."""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
