"""CPU oracle (test infrastructure only): ctypes front for oracle/npas_oracle.c.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this
package.  It never imports the HIP library or its Python binding.
"""
from .api import *  # noqa: F401,F403
