"""CPU oracle -- TEST INFRASTRUCTURE ONLY.

A plain textbook Earley recognizer and the per-step vocabulary mask written out
from its definition.  The product library never imports this package; only the
tests, the smoke check and the benchmark's CPU-baseline leg do.
"""
from .frontend import Oracle, OracleState, desugar, parse_regex, build  # noqa: F401
