"""CPU oracle (test infrastructure only).

Nothing in the product package imports this.  It is loaded by the tests, by the smoke check and
by the CPU-baseline leg of the benchmark.
"""
from .oracle_lib import Oracle, build_oracle, oracle_lib, qr_pool  # noqa: F401
