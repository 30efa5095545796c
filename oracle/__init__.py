"""CPU oracle (fp64) of the rotated-shard linear layer.  Test infrastructure
only: nothing on the product path may import this package."""
from .rtp_oracle import *  # noqa: F401,F403
from . import rtp_oracle as _impl

__all__ = [n for n in dir(_impl) if not n.startswith("_")]
