"""CPU oracle of the SAP-scheduled Lasso round.  Test infrastructure only:
imported by tests/, the smoke check and bench.py's cpu_baseline leg."""
from .oracle import OracleLasso, build, lib  # noqa: F401
