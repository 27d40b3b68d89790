"""CPU oracle for the QODA hot path -- test infrastructure, not the product.

Only tests, the smoke check and the bench's cpu_baseline leg import this package.  It wraps
``qoda_oracle.cpp`` (plain single-threaded C++) through ctypes and adds nothing to its arithmetic:
every function here marshals numpy arrays and calls one oracle routine.
"""
from .oracle import *  # noqa: F401,F403
from .oracle import build  # noqa: F401
