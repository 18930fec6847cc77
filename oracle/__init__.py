"""CPU oracle for the HEART hot path -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
package.  It compiles `heart_oracle.c` with gcc (plain C + OpenMP, fp64
accumulation) and exposes thin numpy wrappers; it imports nothing from the HIP
package and the HIP package imports nothing from here.
"""
from .heart_oracle import (  # noqa: F401
    build,
    pool,
    drift,
    scores,
    topp,
    attn,
    dense_attn,
    num_threads,
)
from . import ebc_oracle  # noqa: F401
from . import antidiag_oracle  # noqa: F401
