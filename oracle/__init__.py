"""CPU oracle for the context-switch swap.  TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Only tests, the smoke check and the bench's ``cpu_baseline`` leg may import this
package.  It shares nothing with the GPU library and never imports it.
"""
from .nixie_oracle import (  # noqa: F401
    Oracle, OracleError, build, FAULTS, lib_path,
)
from .sched_oracle import SchedOracle  # noqa: F401,E402
from . import place_oracle  # noqa: F401,E402
