"""CPU oracle: test infrastructure only (tests, the smoke check, the benchmark's CPU baseline)."""
from .cpu import ingest, evaluate, evaluate_parallel, evaluate_ticks, mixed, select_path, account, hierarchy, window_totals, select_row  # noqa: F401
