"""fp64 CPU oracle for RACE Attention.  Test infrastructure: never imported by the product path.

race_oracle         numpy: the N x N definition, Algorithms 1 and 2 as written, the derived
                    backward in quadratic and streaming form, finite differences, and the
                    seed -> W generator.
stream              ctypes front end of race_oracle_stream.c: the same linear-time algorithms in
                    plain C/OpenMP, for sequence lengths the numpy loops cannot reach.
"""
from . import race_oracle  # noqa: F401
from . import stream  # noqa: F401
