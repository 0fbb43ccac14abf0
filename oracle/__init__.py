"""CPU oracle of the stage hot path.  TEST INFRASTRUCTURE ONLY: imported by tests/, by
__graft_entry__.smoke() and by bench.py's cpu_baseline leg, never by the product path."""
from .stage import OracleStage, build, gcn_norm, max_threads, set_threads  # noqa: F401
