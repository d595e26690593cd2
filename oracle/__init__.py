"""CPU checker for the decoder -- TEST INFRASTRUCTURE, not product code.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this
package.  It shares nothing with the HIP library.
"""
from .oracle import (OracleGraph, OracleChannel, build_oracle, prune,  # noqa: F401
                     ORC_OK, ORC_NO_TOKENS, ORC_EPS_DIVERGED)
from .word_arcs import arcs_for_sequence, arcs_for_sequences  # noqa: F401
