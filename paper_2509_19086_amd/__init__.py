"""MI355X-native batched gap-job fit evaluation and slot grant.

`Engine` wraps the C-ABI library (libsja.so, hand-written HIP for gfx950); the
methods carry the same names as the C entry points declared in include/sja.h.
"""
from .binding import (  # noqa: F401
    Engine, Params, Limits, SjaError, load_library,
    POLICY_EFFICIENCY, POLICY_FAIRNESS, POLICY_SLA, POLICY_MIXED,
)
from .tick import DeviceTick  # noqa: F401
