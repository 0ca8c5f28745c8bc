"""Conf-KV per-decode-step hot path for AMD MI355X: HIP library + thin ctypes binding."""
from .binding import (ConfKV, ConfKVConfig, ConfKVError, ConfKVStats, LIB_PATH, SYMBOLS,  # noqa: F401
                      from_workload, load_library, make_config, probe_read, pyramid_budgets, strerror)
