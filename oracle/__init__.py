"""CPU oracle for DeepPoly back-substitution.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this package.
The HIP library and its Python binding never do.
"""
from .deeppoly import OracleNet, build_oracle, oracle_threads  # noqa: F401
