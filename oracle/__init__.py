"""fp64 CPU oracle of the verification hot path.  Test infrastructure only:
importable from tests/, the smoke check and the benchmark's cpu_baseline leg."""
from .specext_oracle import *  # noqa: F401,F403
