"""CPU oracle package (test infrastructure only; see ilargi_oracle.py)."""
from .ilargi_oracle import *  # noqa: F401,F403
from . import ilargi_oracle as _impl

__all__ = [n for n in dir(_impl) if not n.startswith("_")]
