"""CPU oracle for the repetend-candidate evaluator: test infrastructure only.

Nothing in the product path imports this package; tests, the smoke check and the
benchmark's cpu_baseline leg do.
"""
from .oracle import Oracle, OracleScore, OracleResult, build_oracle, STATUS_NAMES  # noqa: F401
