"""fp64 CPU oracle for decode attention (test infrastructure, not the product).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this package.  It never imports the HIP package.
"""
from .ta_oracle import (  # noqa: F401
    decode, decode_causal, energy_causal, partial, combine, combine_alg3, energy, recurrence, two_pass,
    max_threads, flat_merges, as_oracle_array,
)
