"""CPU oracle for HBMM: test infrastructure only (tests, smoke check, cpu_baseline)."""
from .hbmm_oracle import *  # noqa: F401,F403
