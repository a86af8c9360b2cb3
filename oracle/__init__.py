"""CPU oracle for the Tri-Accel optimizer step -- TEST INFRASTRUCTURE ONLY.

The arithmetic lives in ``triaccel_oracle.c`` (plain C, compiled with gcc,
``-ffp-contract=off``); this package compiles it on demand, exposes the C
functions through ctypes on numpy arrays, and sequences them into one
optimizer step (``oracle.step``).  It shares no code with the HIP library and
must never be imported by the product package: only the tests, the smoke check
and the benchmark's CPU-baseline leg use it.
"""

from .capi import build, lib  # noqa: F401
from .step import OracleConfig, OracleTensor, OracleTriAccel  # noqa: F401
