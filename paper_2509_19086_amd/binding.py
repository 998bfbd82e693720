"""Thin ctypes binding over libsja.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels; PyTorch is used for
device memory (tensors) and the current stream.  There is no CPU fallback: if
the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

from . import build as _build

POLICY_EFFICIENCY, POLICY_FAIRNESS, POLICY_SLA, POLICY_MIXED = 0, 1, 2, 3

_lib = None


class SjaError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{text} (status {status})")
        self.status = status


class Params(ctypes.Structure):
    """Mirror of sja_params."""
    _fields_ = [("policy", ctypes.c_int32), ("wait_scale", ctypes.c_int32),
                ("sla_weight", ctypes.c_int32 * 3), ("class0_override", ctypes.c_int32),
                ("max_rounds", ctypes.c_int32)]

    @classmethod
    def make(cls, policy: int, wait_scale: int = 1000, sla_weight: Sequence[int] = (4, 2, 1),
             class0_override: int = 1, max_rounds: int = 0) -> "Params":
        return cls(policy, wait_scale, (ctypes.c_int32 * 3)(*sla_weight), class0_override,
                   max_rounds)


class Limits(ctypes.Structure):
    """Mirror of sja_limits."""
    _fields_ = [("tau_min", ctypes.c_int32), ("tau_max", ctypes.c_int32),
                ("power_cap", ctypes.c_int32), ("now", ctypes.c_int32)]

    @classmethod
    def make(cls, tau_min: int = 0, tau_max: int = 2**31 - 1, power_cap: int = 2**31 - 1,
             now: int = 0) -> "Limits":
        return cls(tau_min, tau_max, power_cap, now)


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Loads the built library.  Builds it only when none is there at all; a library that is
    older than its sources is loaded as it is, with a warning (build again before testing)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or _build.LIB
    if not os.path.exists(p):
        _build.build(force=True)
    elif path is None and _build.is_stale():
        import warnings
        warnings.warn(f"{p} is older than its sources: run `python -m paper_2509_19086_amd.build`")
    if not os.path.exists(p):
        raise FileNotFoundError(f"{p} is missing: run `python -m paper_2509_19086_amd.build`")
    lib = ctypes.CDLL(p)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.sja_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int]
    lib.sja_create.restype = ctypes.c_int
    lib.sja_destroy.argtypes = [vp]
    lib.sja_destroy.restype = ctypes.c_int
    lib.sja_workspace_bytes.argtypes = [i64, i64, i64]
    lib.sja_workspace_bytes.restype = ctypes.c_size_t
    lib.sja_set_workspace.argtypes = [vp, vp, ctypes.c_size_t]
    lib.sja_set_workspace.restype = ctypes.c_int
    lib.sja_status_string.argtypes = [ctypes.c_int]
    lib.sja_status_string.restype = ctypes.c_char_p
    lib.sja_last_error.argtypes = [vp]
    lib.sja_last_error.restype = ctypes.c_char_p
    lib.sja_prepare_profiles.argtypes = [vp, vp, i32, i64] + [vp] * 8
    lib.sja_prepare_profiles.restype = ctypes.c_int
    lib.sja_prepare_profiles_static.argtypes = [vp, vp, i32, i64] + [vp] * 8
    lib.sja_prepare_profiles_static.restype = ctypes.c_int
    lib.sja_fit.argtypes = [vp, vp, i32] + [vp] * 4
    lib.sja_fit.restype = ctypes.c_int
    lib.sja_select.argtypes = [vp, vp, ctypes.POINTER(Params)] + [vp] * 7
    lib.sja_select.restype = ctypes.c_int
    lib.sja_resolve.argtypes = [vp, vp, ctypes.POINTER(Params)] + [vp] * 7
    lib.sja_fit_select.argtypes = [vp, vp, i32, vp, vp, ctypes.POINTER(Params)] + [vp] * 7
    lib.sja_fit_select.restype = ctypes.c_int
    lib.sja_resolve.restype = ctypes.c_int
    lib.sja_set_score.argtypes = [vp, ctypes.c_int]
    lib.sja_set_score.restype = ctypes.c_int
    lib.sja_set_limits.argtypes = [vp, ctypes.POINTER(Limits), vp, vp]
    lib.sja_set_limits.restype = ctypes.c_int
    lib.sja_set_hysteresis.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_int32), i32]
    lib.sja_set_hysteresis.restype = ctypes.c_int
    lib.sja_cover.argtypes = [vp, vp, i32, vp, vp, vp, i32, vp, vp, vp]
    lib.sja_cover.restype = ctypes.c_int
    lib.sja_validate.argtypes = [vp, vp, i32, i64, vp, vp, vp, vp, ctypes.POINTER(Params), vp, vp, vp]
    lib.sja_validate.restype = ctypes.c_int
    lib.sja_advance.argtypes = [vp, vp, i32] + [vp] * 7 + [i32, vp]
    lib.sja_advance.restype = ctypes.c_int
    lib.sja_enable_timing.argtypes = [vp, ctypes.c_int]
    lib.sja_enable_timing.restype = ctypes.c_int
    lib.sja_last_fit_kernel_ms.argtypes = [vp, ctypes.POINTER(ctypes.c_float)]
    lib.sja_last_fit_kernel_ms.restype = ctypes.c_int
    lib.sja_store_reference.argtypes = [vp, vp, vp]
    lib.sja_store_reference.restype = ctypes.c_int
    lib.sja_set_resolve_mode.argtypes = [vp, ctypes.c_int]
    lib.sja_set_resolve_mode.restype = ctypes.c_int
    if path is None:
        _lib = lib
    return lib


def _ptr(t: Optional[torch.Tensor], dtype: torch.dtype, n: Optional[int] = None) -> ctypes.c_void_p:
    if t is None:
        return ctypes.c_void_p(0)
    if not isinstance(t, torch.Tensor) or t.dtype != dtype:
        raise TypeError(f"expected a {dtype} tensor, got {getattr(t, 'dtype', type(t))}")
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors must be contiguous and on the GPU")
    if n is not None and t.numel() < n:
        raise ValueError(f"tensor has {t.numel()} elements, {n} needed")
    return ctypes.c_void_p(t.data_ptr())


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


class Engine:
    """One sja_ctx plus its workspace tensor.  Methods mirror the C entry points."""

    def __init__(self, device: int = 0):
        self.lib = load_library()
        self.device = device
        h = ctypes.c_void_p()
        self._check(self.lib.sja_create(ctypes.byref(h), device), None)
        self.h = h
        self.workspace: Optional[torch.Tensor] = None
        self.n_jobs = 0
        self.n_gaps = 0

    def close(self) -> None:
        if getattr(self, "h", None):
            self.lib.sja_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int, h) -> None:
        if rc != 0:
            text = self.lib.sja_last_error(h).decode() if h else self.lib.sja_status_string(rc).decode()
            raise SjaError(rc, text)

    def workspace_bytes(self, n_gaps: int, n_jobs: int, n_segments: int) -> int:
        return int(self.lib.sja_workspace_bytes(n_gaps, n_jobs, n_segments))

    def ensure_workspace(self, n_gaps: int, n_jobs: int, n_segments: int) -> None:
        need = self.workspace_bytes(n_gaps, n_jobs, n_segments)
        if need == 0 and (n_gaps or n_jobs or n_segments):
            raise SjaError(-2, "sizes beyond the library's limits")
        if self.workspace is None or self.workspace.numel() < need:
            self.workspace = torch.empty(max(need, 256), dtype=torch.uint8,
                                         device=f"cuda:{self.device}")
            self._check(self.lib.sja_set_workspace(self.h, ctypes.c_void_p(self.workspace.data_ptr()),
                                                   self.workspace.numel()), self.h)

    def sja_enable_timing(self, on: bool) -> None:
        self._check(self.lib.sja_enable_timing(self.h, int(on)), self.h)

    def sja_store_reference(self, cut) -> None:
        """Overwrites cut [n_gaps, n_jobs] with the pair-evaluation kernel's store stream (cut[g][j] = j)."""
        self._check(self.lib.sja_store_reference(self.h, _stream(), _ptr(cut, torch.int32, self.n_gaps * self.n_jobs)),
                    self.h)

    def sja_set_resolve_mode(self, mode: int) -> None:
        """0 = candidate lists (default), 1 = matrix-scanning rounds."""
        self._check(self.lib.sja_set_resolve_mode(self.h, int(mode)), self.h)

    def sja_last_fit_kernel_ms(self) -> float:
        ms = ctypes.c_float()
        self._check(self.lib.sja_last_fit_kernel_ms(self.h, ctypes.byref(ms)), self.h)
        return float(ms.value)

    # -- the four calls --------------------------------------------------
    def sja_prepare_profiles(self, seg_off, dur, mem, safe, progress, pre_dur, pre_peak, prev_safe,
                             _entry="sja_prepare_profiles"):
        J = seg_off.numel() - 1
        S = dur.numel()
        args = (_ptr(seg_off, torch.int64, J + 1), _ptr(dur, torch.int32, S),
                _ptr(mem, torch.int32, S), _ptr(safe, torch.uint8, S), _ptr(progress, torch.int32, J),
                _ptr(pre_dur, torch.int32, S), _ptr(pre_peak, torch.int32, S),
                _ptr(prev_safe, torch.int32, S))
        rc = getattr(self.lib, _entry)(self.h, _stream(), J, S, *args)
        self._check(rc, self.h)
        self.n_jobs = J
        self.n_gaps = 0          # a new prepare ends the last batch of gaps, as in the library

    def sja_prepare_profiles_static(self, seg_off, dur, mem, safe, progress, pre_dur, pre_peak, prev_safe):
        """The same call on the library's built-in scratch: no workspace tensor is involved."""
        self.sja_prepare_profiles(seg_off, dur, mem, safe, progress, pre_dur, pre_peak, prev_safe,
                                  _entry="sja_prepare_profiles_static")

    def sja_fit(self, W, C, cut, interest_bits=None):
        G = W.numel()
        words = (self.n_jobs + 31) // 32
        args = (_ptr(W, torch.int32, G), _ptr(C, torch.int32, G),
                _ptr(cut, torch.int32, G * self.n_jobs), _ptr(interest_bits, torch.int32, G * words))
        rc = self.lib.sja_fit(self.h, _stream(), G, *args)
        self._check(rc, self.h)
        self.n_gaps = G

    def sja_fit_select(self, W, C, params: Params, wait, sla_class, job_held, gap_active,
                       cand_job, cand_cut, cand_score):
        G, J = W.numel(), self.n_jobs
        args = (_ptr(W, torch.int32, G), _ptr(C, torch.int32, G))
        rest = (_ptr(wait, torch.int32, J), _ptr(sla_class, torch.uint8, J),
                _ptr(job_held, torch.int32, J), _ptr(gap_active, torch.uint8, G),
                _ptr(cand_job, torch.int32, G), _ptr(cand_cut, torch.int32, G),
                _ptr(cand_score, torch.int64, G))
        rc = self.lib.sja_fit_select(self.h, _stream(), G, *args, ctypes.byref(params), *rest)
        self._check(rc, self.h)
        self.n_gaps = G

    def sja_select(self, params: Params, wait, sla_class, job_held, gap_active,
                   cand_job, cand_cut, cand_score):
        G, J = self.n_gaps, self.n_jobs
        args = (_ptr(wait, torch.int32, J), _ptr(sla_class, torch.uint8, J),
                _ptr(job_held, torch.int32, J), _ptr(gap_active, torch.uint8, G),
                _ptr(cand_job, torch.int32, G), _ptr(cand_cut, torch.int32, G),
                _ptr(cand_score, torch.int64, G))
        rc = self.lib.sja_select(self.h, _stream(), ctypes.byref(params), *args)
        self._check(rc, self.h)

    def sja_resolve(self, params: Params, wait, sla_class, grant_job, grant_cut, grant_score,
                    job_gap, rounds_used_and_stable):
        G, J = self.n_gaps, self.n_jobs
        args = (_ptr(wait, torch.int32, J), _ptr(sla_class, torch.uint8, J),
                _ptr(grant_job, torch.int32, G), _ptr(grant_cut, torch.int32, G),
                _ptr(grant_score, torch.int64, G), _ptr(job_gap, torch.int32, J),
                _ptr(rounds_used_and_stable, torch.int32, 2))
        rc = self.lib.sja_resolve(self.h, _stream(), ctypes.byref(params), *args)
        self._check(rc, self.h)

    def sja_validate(self, seg_off, dur, mem, progress, params, wait, sla_class, problems):
        J, S = seg_off.numel() - 1, dur.numel()
        rc = self.lib.sja_validate(self.h, _stream(), J, S, _ptr(seg_off, torch.int64, J + 1),
                                   _ptr(dur, torch.int32, S), _ptr(mem, torch.int32, S),
                                   _ptr(progress, torch.int32, J),
                                   ctypes.byref(params) if params is not None else None,
                                   _ptr(wait, torch.int32, J), _ptr(sla_class, torch.uint8, J),
                                   _ptr(problems, torch.int32, 1))
        self._check(rc, self.h)

    def sja_set_score(self, score: int) -> None:
        self._check(self.lib.sja_set_score(self.h, int(score)), self.h)

    def sja_set_limits(self, limits, power=None, deadline=None):
        """limits: a Limits or None (clear).  power / deadline: device int32 tensors or None;
        the engine keeps them alive until the limits are replaced."""
        self._limit_arrays = (power, deadline)
        rc = self.lib.sja_set_limits(self.h, ctypes.byref(limits) if limits is not None else None,
                                     _ptr(power, torch.int32), _ptr(deadline, torch.int32))
        self._check(rc, self.h)

    def sja_set_hysteresis(self, cap_set, min_gain: int = 1) -> None:
        """cap_set: a host sequence of ascending capacities (empty or None switches the rule off)."""
        caps = [int(c) for c in (cap_set if cap_set is not None else [])]
        arr = (ctypes.c_int32 * max(len(caps), 1))(*caps)
        self._check(self.lib.sja_set_hysteresis(self.h, len(caps), arr, int(min_gain)), self.h)

    def sja_cover(self, C, grant_job, grant_cut, cap_set, cover, slack):
        G, K = C.numel(), cap_set.numel()
        args = (_ptr(C, torch.int32, G), _ptr(grant_job, torch.int32, G), _ptr(grant_cut, torch.int32, G))
        rc = self.lib.sja_cover(self.h, _stream(), G, *args, K, _ptr(cap_set, torch.int32, K),
                                _ptr(cover, torch.int32, G), _ptr(slack, torch.int32, G))
        self._check(rc, self.h)

    def sja_advance(self, W, C, grant_job, grant_cut, job_gap, progress, wait, wait_step, metrics):
        G, J = W.numel(), self.n_jobs
        args = (_ptr(W, torch.int32, G), _ptr(C, torch.int32, G), _ptr(grant_job, torch.int32, G),
                _ptr(grant_cut, torch.int32, G), _ptr(job_gap, torch.int32, J),
                _ptr(progress, torch.int32, J), _ptr(wait, torch.int32, J))
        rc = self.lib.sja_advance(self.h, _stream(), G, *args, int(wait_step), _ptr(metrics, torch.int64, 4))
        self._check(rc, self.h)
