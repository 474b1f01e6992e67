"""Float64 CPU oracle of the VQ decode-attention path.  Test infrastructure only."""
from .oracle import *  # noqa: F401,F403
from . import oracle as _o

build = _o.build
