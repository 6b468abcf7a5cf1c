"""CPU oracle for the decode step (test infrastructure only).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this package.  It never imports the HIP path and the HIP path never imports
it.  The arithmetic lives in decode_oracle.c; this file compiles it with gcc
and marshals numpy arrays into it.
"""
from .reference import (  # noqa: F401
    build, Oracle, oracle_f64, oracle_f32,
)
