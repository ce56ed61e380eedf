"""CPU oracle (test infrastructure; see interp.py).  Never imported by the product path."""
from .interp import run, run_outputs, OracleError  # noqa: F401
