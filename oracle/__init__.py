"""CPU oracle for the plan-search dynamic program — TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package.  The product path (the HIP library and its binding) never does.

  * ``solve``        — the serial C implementation (galv_oracle.c) of the layer
                       recurrence of paper section 3.3, Eq. 1.
  * ``brute_force``  — the plain definition: enumerate every plan (bruteforce.py).
"""
from .binding import INF, OracleResult, build, solve, solve_workload  # noqa: F401
from .bruteforce import brute_force, brute_force_cells  # noqa: F401
