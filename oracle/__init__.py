"""fp64 CPU oracle for the SPECTRE mixer and Prefix-FFT cache.

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the
CPU-baseline leg of the benchmark.  The GPU library and its Python binding never
import this package, and this package never imports them.
"""
from .spectre_oracle import *  # noqa: F401,F403
