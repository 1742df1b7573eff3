"""CPU oracle for the MGRIT transformer-ODE hot path.

TEST INFRASTRUCTURE ONLY: slow, plain, float64 numpy written from the paper.
It shares no code with the HIP library and must never be imported by the
product package; only tests, the smoke check and the benchmark's cpu_baseline
leg use it.
"""
from . import transformer_ode, mgrit  # noqa: F401
