"""TEST INFRASTRUCTURE: ctypes wrapper around oracle/sja_oracle.c.

Argument marshalling only -- every number comes out of the C file.  The
shared object is compiled with gcc on first use (and by the repository's
build step); nothing here is reachable from the GPU library or its binding.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

POLICY_EFFICIENCY, POLICY_FAIRNESS, POLICY_SLA, POLICY_MIXED = 0, 1, 2, 3

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sja_oracle.c")
_LIB = os.path.join(_HERE, "libsja_oracle.so")
_lib = None


def lib_path() -> str:
    return _LIB


def build(force: bool = False) -> str:
    """Compile the oracle (gcc -O2, OpenMP over the outer gap loops)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
        global _lib
        _lib = None
    return _LIB


class Params(ctypes.Structure):
    _fields_ = [("policy", ctypes.c_int32), ("wait_scale", ctypes.c_int32),
                ("sla_weight", ctypes.c_int32 * 3), ("class0_override", ctypes.c_int32),
                ("max_rounds", ctypes.c_int32)]

    @classmethod
    def make(cls, policy: int, wait_scale: int = 1000, sla_weight: Sequence[int] = (4, 2, 1),
             class0_override: int = 1, max_rounds: int = 0) -> "Params":
        return cls(policy, wait_scale, (ctypes.c_int32 * 3)(*sla_weight), class0_override,
                   max_rounds)


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.sjo_num_threads.restype = ctypes.c_int
        for name in ("sjo_prepare", "sjo_fit", "sjo_fit_pairs", "sjo_select", "sjo_resolve"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().sjo_num_threads())


def set_num_threads(n: int) -> None:
    _load().sjo_set_num_threads(ctypes.c_int(n))


def _p(a: Optional[np.ndarray], dtype) -> ctypes.c_void_p:
    if a is None:
        return ctypes.c_void_p(0)
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags.c_contiguous, \
        (getattr(a, "dtype", None), dtype)
    return ctypes.c_void_p(a.ctypes.data)


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise RuntimeError(f"{what} failed with oracle status {rc}")


def prepare(seg_off, dur, mem, safe, progress, fill: int = -7):
    """Returns (pre_dur int64, pre_peak int64, prev_safe int32); untouched entries = fill."""
    J = len(seg_off) - 1
    S = int(seg_off[-1])
    pre_dur = np.full(S, fill, dtype=np.int64)
    pre_peak = np.full(S, fill, dtype=np.int64)
    prev_safe = np.full(S, fill, dtype=np.int32)
    rc = _load().sjo_prepare(ctypes.c_int32(J), _p(seg_off, np.int64), _p(dur, np.int32),
                             _p(mem, np.int32), _p(safe, np.uint8), _p(progress, np.int32),
                             _p(pre_dur, np.int64), _p(pre_peak, np.int64),
                             _p(prev_safe, np.int32))
    _check(rc, "sjo_prepare")
    return pre_dur, pre_peak, prev_safe


def area(seg_off, dur, mem, progress, fill: int = -7):
    """pre_area int64 [S]: area under the envelope from each job's progress point; untouched = fill."""
    J = len(seg_off) - 1
    out = np.full(int(seg_off[-1]), fill, dtype=np.int64)
    rc = _load().sjo_area(ctypes.c_int32(J), _p(seg_off, np.int64), _p(dur, np.int32), _p(mem, np.int32),
                          _p(progress, np.int32), _p(out, np.int64))
    _check(rc, "sjo_area")
    return out


class Limits(ctypes.Structure):
    """Mirror of sjo_limits (admission limits of Sec. 4.3 / 4.4)."""
    _fields_ = [("tau_min", ctypes.c_int32), ("tau_max", ctypes.c_int32),
                ("power_cap", ctypes.c_int32), ("now", ctypes.c_int32)]

    @classmethod
    def make(cls, tau_min: int = 0, tau_max: int = 2**31 - 1, power_cap: int = 2**31 - 1, now: int = 0):
        return cls(tau_min, tau_max, power_cap, now)


def fit_limited(seg_off, dur, mem, safe, progress, W, C, limits, power=None, deadline=None,
                want_bits: bool = False):
    """fit() under admission limits: returns (cut [G, J] int32, bits or None)."""
    G, J = len(W), len(seg_off) - 1
    cut = np.empty((G, J), dtype=np.int32)
    bits = np.zeros((G, (J + 31) // 32), dtype=np.uint32) if want_bits else None
    rc = _load().sjo_fit_limited(ctypes.c_int32(G), ctypes.c_int32(J), _p(seg_off, np.int64),
                                 _p(dur, np.int32), _p(mem, np.int32), _p(safe, np.uint8),
                                 _p(progress, np.int32), _p(W, np.int32), _p(C, np.int32),
                                 ctypes.byref(limits) if limits is not None else None,
                                 _p(power, np.int32), _p(deadline, np.int32), _p(cut, np.int32),
                                 _p(bits, np.uint32))
    _check(rc, "sjo_fit_limited")
    return cut, bits


def fit_pairs_limited(gap_idx, job_idx, seg_off, dur, mem, safe, progress, W, C, limits, power=None,
                      deadline=None):
    """fit_pairs() under admission limits; returns (cut int32, sub_dur int64, sub_peak int64)."""
    n = len(gap_idx)
    cut = np.empty(n, dtype=np.int32)
    sd = np.empty(n, dtype=np.int64)
    sp = np.empty(n, dtype=np.int64)
    rc = _load().sjo_fit_pairs_limited(ctypes.c_int64(n), _p(gap_idx, np.int32), _p(job_idx, np.int32),
                                       _p(seg_off, np.int64), _p(dur, np.int32), _p(mem, np.int32),
                                       _p(safe, np.uint8), _p(progress, np.int32), _p(W, np.int32),
                                       _p(C, np.int32),
                                       ctypes.byref(limits) if limits is not None else None,
                                       _p(power, np.int32), _p(deadline, np.int32), _p(cut, np.int32),
                                       _p(sd, np.int64), _p(sp, np.int64))
    _check(rc, "sjo_fit_pairs_limited")
    return cut, sd, sp


def fit_hysteresis(seg_off, dur, mem, safe, progress, W, C, cap_set, min_gain, limits=None, power=None,
                   deadline=None, want_bits: bool = False):
    """fit_limited() under the hysteresis rule of Sec. 3.9 (cap_set ascending, min_gain >= 1):
    returns (cut [G, J] int32, bits or None)."""
    G, J = len(W), len(seg_off) - 1
    cap_set = np.ascontiguousarray(cap_set, dtype=np.int32)
    cut = np.empty((G, J), dtype=np.int32)
    bits = np.zeros((G, (J + 31) // 32), dtype=np.uint32) if want_bits else None
    rc = _load().sjo_fit_hysteresis(ctypes.c_int32(G), ctypes.c_int32(J), _p(seg_off, np.int64),
                                    _p(dur, np.int32), _p(mem, np.int32), _p(safe, np.uint8),
                                    _p(progress, np.int32), _p(W, np.int32), _p(C, np.int32),
                                    ctypes.byref(limits) if limits is not None else None,
                                    _p(power, np.int32), _p(deadline, np.int32),
                                    ctypes.c_int32(len(cap_set)), _p(cap_set, np.int32),
                                    ctypes.c_int32(min_gain), _p(cut, np.int32), _p(bits, np.uint32))
    _check(rc, "sjo_fit_hysteresis")
    return cut, bits


def fit_pairs_hysteresis(gap_idx, job_idx, seg_off, dur, mem, safe, progress, W, C, cap_set, min_gain,
                         limits=None, power=None, deadline=None):
    """fit_hysteresis() on sampled pairs; returns (cut int32, sub_dur int64, sub_peak int64)."""
    n = len(gap_idx)
    cap_set = np.ascontiguousarray(cap_set, dtype=np.int32)
    cut = np.empty(n, dtype=np.int32)
    sd = np.empty(n, dtype=np.int64)
    sp = np.empty(n, dtype=np.int64)
    rc = _load().sjo_fit_pairs_hysteresis(ctypes.c_int64(n), _p(gap_idx, np.int32), _p(job_idx, np.int32),
                                          _p(seg_off, np.int64), _p(dur, np.int32), _p(mem, np.int32),
                                          _p(safe, np.uint8), _p(progress, np.int32), _p(W, np.int32),
                                          _p(C, np.int32),
                                          ctypes.byref(limits) if limits is not None else None,
                                          _p(power, np.int32), _p(deadline, np.int32),
                                          ctypes.c_int32(len(cap_set)), _p(cap_set, np.int32),
                                          ctypes.c_int32(min_gain), _p(cut, np.int32), _p(sd, np.int64),
                                          _p(sp, np.int64))
    _check(rc, "sjo_fit_pairs_hysteresis")
    return cut, sd, sp


def cover(seg_off, pre_peak, C, grant_job, grant_cut, cap_set):
    """Smallest capacity of cap_set (ascending) covering each grant's peak, and the slack
    against the gap's own capacity: (cover int32 [G], slack int32 [G])."""
    G = len(C)
    cap_set = np.ascontiguousarray(cap_set, dtype=np.int32)
    cov = np.empty(G, dtype=np.int32)
    slack = np.empty(G, dtype=np.int32)
    rc = _load().sjo_cover(ctypes.c_int32(G), _p(seg_off, np.int64), _p(pre_peak, np.int64),
                           _p(C, np.int32), _p(grant_job, np.int32), _p(grant_cut, np.int32),
                           ctypes.c_int32(len(cap_set)), _p(cap_set, np.int32), _p(cov, np.int32),
                           _p(slack, np.int32))
    _check(rc, "sjo_cover")
    return cov, slack


def fit(seg_off, dur, mem, safe, progress, W, C, want_bits: bool = True):
    """Returns (cut int32 [G, J], interest_bits uint32 [G, ceil(J/32)] or None)."""
    J = len(seg_off) - 1
    G = len(W)
    cut = np.empty((G, J), dtype=np.int32)
    bits = np.empty((G, (J + 31) // 32), dtype=np.uint32) if want_bits else None
    rc = _load().sjo_fit(ctypes.c_int32(G), ctypes.c_int32(J), _p(seg_off, np.int64),
                         _p(dur, np.int32), _p(mem, np.int32), _p(safe, np.uint8),
                         _p(progress, np.int32), _p(W, np.int32), _p(C, np.int32),
                         _p(cut, np.int32), _p(bits, np.uint32))
    _check(rc, "sjo_fit")
    return cut, bits


def fit_pairs(gap_idx, job_idx, seg_off, dur, mem, safe, progress, W, C):
    """Fit on sampled pairs; returns (cut int32, sub_dur int64, sub_peak int64)."""
    n = len(gap_idx)
    gap_idx = np.ascontiguousarray(gap_idx, dtype=np.int32)
    job_idx = np.ascontiguousarray(job_idx, dtype=np.int32)
    cut = np.empty(n, dtype=np.int32)
    sd = np.empty(n, dtype=np.int64)
    sp = np.empty(n, dtype=np.int64)
    rc = _load().sjo_fit_pairs(ctypes.c_int64(n), _p(gap_idx, np.int32), _p(job_idx, np.int32),
                               _p(seg_off, np.int64), _p(dur, np.int32), _p(mem, np.int32),
                               _p(safe, np.uint8), _p(progress, np.int32), _p(W, np.int32),
                               _p(C, np.int32), _p(cut, np.int32), _p(sd, np.int64),
                               _p(sp, np.int64))
    _check(rc, "sjo_fit_pairs")
    return cut, sd, sp


def select(cut, seg_off, pre_dur, pre_peak, params: Params, wait, sla_class,
           job_held=None, gap_active=None, pre_area=None):
    """Returns (cand_job int32 [G], cand_cut int32 [G], cand_score int64 [G]).
    pre_area (from area()) scores by the area under the envelope instead of duration x peak."""
    G, J = cut.shape
    cj = np.empty(G, dtype=np.int32)
    cc = np.empty(G, dtype=np.int32)
    cs = np.empty(G, dtype=np.int64)
    rc = _load().sjo_select(ctypes.c_int32(G), ctypes.c_int32(J), _p(cut, np.int32),
                            _p(seg_off, np.int64), _p(pre_dur, np.int64), _p(pre_peak, np.int64),
                            _p(pre_area, np.int64),
                            ctypes.byref(params), _p(wait, np.int32), _p(sla_class, np.uint8),
                            _p(job_held, np.int32), _p(gap_active, np.uint8),
                            _p(cj, np.int32), _p(cc, np.int32), _p(cs, np.int64))
    _check(rc, "sjo_select")
    return cj, cc, cs


def resolve(cut, seg_off, pre_dur, pre_peak, params: Params, wait, sla_class, pre_area=None):
    """Returns (grant_job, grant_cut, grant_score, job_gap, rounds_used, stable)."""
    G, J = cut.shape
    gj = np.empty(G, dtype=np.int32)
    gc = np.empty(G, dtype=np.int32)
    gs = np.empty(G, dtype=np.int64)
    jg = np.empty(J, dtype=np.int32)
    rs = np.zeros(2, dtype=np.int32)
    rc = _load().sjo_resolve(ctypes.c_int32(G), ctypes.c_int32(J), _p(cut, np.int32),
                             _p(seg_off, np.int64), _p(pre_dur, np.int64),
                             _p(pre_peak, np.int64), _p(pre_area, np.int64), ctypes.byref(params),
                             _p(wait, np.int32),
                             _p(sla_class, np.uint8), _p(gj, np.int32), _p(gc, np.int32),
                             _p(gs, np.int64), _p(jg, np.int32), _p(rs, np.int32))
    _check(rc, "sjo_resolve")
    return gj, gc, gs, jg, int(rs[0]), int(rs[1])


def advance(seg_off, pre_dur, pre_peak, W, C, grant_job, grant_cut, job_gap, progress, wait, wait_step):
    """Next tick's (progress, wait) and the tick's metrics (filled, offered, grants, finished).
    progress and wait are copied, not changed in place; wait may be None."""
    G, J = len(W), len(seg_off) - 1
    prog = np.array(progress, dtype=np.int32, copy=True)
    wt = None if wait is None else np.array(wait, dtype=np.int32, copy=True)
    metrics = np.zeros(4, dtype=np.int64)
    rc = _load().sjo_advance(ctypes.c_int32(G), ctypes.c_int32(J), _p(seg_off, np.int64),
                             _p(pre_dur, np.int64), _p(pre_peak, np.int64), _p(W, np.int32),
                             _p(C, np.int32), _p(grant_job, np.int32), _p(grant_cut, np.int32),
                             _p(job_gap, np.int32), _p(prog, np.int32),
                             _p(wt, np.int32) if wt is not None else None,
                             ctypes.c_int32(wait_step), _p(metrics, np.int64))
    _check(rc, "sjo_advance")
    return prog, wt, metrics

