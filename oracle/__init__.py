"""CPU oracle: plain, slow, obviously-correct fp64 implementations.

TEST INFRASTRUCTURE ONLY.  Only tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this package.  It shares nothing with the HIP
path and never imports the product package.

Modules: ``ops`` (single operators, C via ctypes), ``models`` (operator
chains with bf16 rounding at the GPU graph's bf16 edges), ``atoms``
(atom-decomposition model), ``rightsize`` (selection rules and the two-point
scaling model), ``sched_sim`` (discrete-event scheduler model).

Parity pins: every function is pinned by tests/test_oracle_*.py against
closed forms, identities, brute force on tiny inputs or an independent
library routine; none is "parity unpinned".
"""
