"""CPU oracle of the GPU embedding cache.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this package.
It imports nothing from the HIP package and shares no code with it.
"""
from .hps_oracle import (OracleCache, mix64, set_of, dedup, expand, load_library,  # noqa: F401
                         EMPTY_KEY, RESERVED_KEY)
