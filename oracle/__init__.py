"""CPU oracle of the filtered exhaustive top-k path -- test infrastructure only.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It never imports the HIP library or its Python binding.
"""
from .linr_oracle import (build, search, pairs, dot_f64, passes, FILTER_DTYPE, NO_ID,  # noqa: F401
                          F32, BF16, I8, widen, sign_oporp, bit_matches, bits_search, two_stage, filter_passes, bits_select,
                          clause_feasible, clause_search)
from .linr_oracle_live import LiveIndex  # noqa: F401
