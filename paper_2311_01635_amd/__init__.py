"""Rotated-shard linear layer of Rotated Tensor Parallelism for one MI355X worker.

`binding` mirrors the C ABI of include/rtp.h one to one; `layers` packs full
matrices into the ring store and owns the torch buffers the library works on.
Importing this package loads librtp.so and raises if it has not been built.
"""
from . import binding  # noqa: F401  (raises when the library is missing)
from .binding import *  # noqa: F401,F403
from .layers import RtpLinear, RtpMlp  # noqa: F401
