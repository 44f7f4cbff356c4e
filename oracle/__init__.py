"""CPU oracle of the BATQuant W4A4 MXFP4 linear hot path.

Test infrastructure: imported only by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports it.
"""
from .batq_oracle import *  # noqa: F401,F403
from . import batq_oracle  # noqa: F401
