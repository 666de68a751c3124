"""CPU oracle for the W4A8 (dINT4 x INT8) linear layer -- TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this package.  It never imports the GPU package and shares no code with it.
"""
from .w4a8_oracle import *  # noqa: F401,F403
from . import aqas_search  # noqa: F401,E402
from . import formats  # noqa: F401,E402
