"""TEST INFRASTRUCTURE ONLY: fp64 CPU oracle for TTT attention.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this package; the GPU
library never does.
"""
from .ttt_oracle import build_oracle, oracle_run, oracle_full, oracle_mask, OracleResult  # noqa: F401
from .ttt_dense import dense_mask_alg2, dense_forward_backward  # noqa: F401
