"""CPU checker (test infrastructure). Only tests, the smoke check and the bench's cpu_baseline leg import this."""
from .oracle import (spgemm_rows, spgemm, build, max_threads, OracleResult, unfold, spttm, fold,  # noqa: F401
                     unfold_mode3, spttm_mode3)
