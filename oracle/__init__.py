"""TEST INFRASTRUCTURE: plain CPU oracle (C, int64) and its ctypes wrapper.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package.  It shares nothing with the GPU path.
"""
from .sja_oracle import (  # noqa: F401
    Params, build, lib_path, num_threads, set_num_threads,
    prepare, fit, fit_pairs, select, resolve, advance,
    Limits, fit_limited, fit_pairs_limited, cover, area, fit_hysteresis, fit_pairs_hysteresis,
    POLICY_EFFICIENCY, POLICY_FAIRNESS, POLICY_SLA, POLICY_MIXED,
)
