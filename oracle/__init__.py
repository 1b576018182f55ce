"""TopLoc CPU oracle: test infrastructure only.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package.  The GPU library never does.
"""
from .toploc_oracle import *  # noqa: F401,F403
