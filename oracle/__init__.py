"""Test infrastructure: the fp64 CPU oracle (see fdc_oracle.py).  Not part of the product path."""
from .fdc_oracle import *  # noqa: F401,F403
from . import fdc_oracle  # noqa: F401
