"""CPU oracle for the walk + SGNS path.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the CPU-baseline leg of the benchmark may
import this package; the product package never does, and this package never
imports the product package.  See ``gs_oracle.cpp`` for what is computed.
"""
from .binding import (  # noqa: F401
    F32, BF16, F16, SYMMETRIZE, DROP_SELF_LOOPS, DEDUPE,
    build, philox4x32_10, csr_build, alias_build, random_walk, node2vec_walk,
    make_pairs, sample_negatives, sample_edges, sgns_step, sgns_momentum_step,
    unique_ids, get_rows, put_rows, sgns_adam_step, line1_step, table_mult, table_mult_add, sort_pairs, f16_to_float, float_to_f16,
)
