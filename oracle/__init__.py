"""CPU oracle (test infrastructure): build + ctypes/numpy wrappers.

Only the tests, the smoke check and the benchmark's cpu_baseline leg import
this package.  It never imports the HIP library's package.
"""
from .api import *  # noqa: F401,F403
