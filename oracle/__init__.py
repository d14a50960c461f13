"""CPU oracle for the SAGE hot path (test infrastructure only).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may import this
package. It shares no code with the HIP library and never calls it.
"""
from .oracle import (Oracle, build_oracle, hestenes_rows, sym_jacobi, topm_f32, keep_count, oracle_threads,  # noqa: F401
                     cb_alpha, cb_budgets, cb_select_from_alpha, cb_scores_and_selection, last_layer_rows, row_dot)
