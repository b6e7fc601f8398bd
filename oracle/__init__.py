"""CPU oracle for the MoE-layer hot path.  TEST INFRASTRUCTURE ONLY.

Only the test-suite, the smoke check and the benchmark's ``cpu_baseline`` leg
may import this package.  It shares no code with the GPU library and never
imports it.
"""
from .moe_oracle import *  # noqa: F401,F403
