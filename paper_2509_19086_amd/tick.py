"""Device-side buffers for one scheduling tick (allocation and upload only)."""
from __future__ import annotations

import numpy as np
import torch

from .binding import Engine, Params


class DeviceTick:
    """Uploads a workload's arrays, allocates every output, and calls the engine.

    `wl` is any object with numpy attributes seg_off, dur, mem, safe, progress,
    W, C, wait, sla_class (see gen.workloads.Workload)."""

    def __init__(self, engine: Engine, wl, want_bits: bool = True, want_cut: bool = True):
        dev = f"cuda:{engine.device}"
        self.engine = engine
        self.G, self.J, self.S = int(len(wl.W)), int(len(wl.seg_off) - 1), int(wl.seg_off[-1])
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        self.seg_off, self.dur, self.mem = up(wl.seg_off), up(wl.dur), up(wl.mem)
        self.safe, self.progress = up(wl.safe), up(wl.progress)
        self.W, self.C = up(wl.W), up(wl.C)
        self.wait, self.sla_class = up(wl.wait), up(wl.sla_class)
        i32 = dict(dtype=torch.int32, device=dev)
        self.pre_dur = torch.full((self.S,), -7, **i32)
        self.pre_peak = torch.full((self.S,), -7, **i32)
        self.prev_safe = torch.full((self.S,), -7, **i32)
        self.cut = torch.empty((self.G, self.J), **i32) if want_cut else None
        self.words = (self.J + 31) // 32
        self.bits = torch.empty((self.G, self.words), **i32) if (want_bits and want_cut) else None
        self.cand_job = torch.empty(self.G, **i32)
        self.cand_cut = torch.empty(self.G, **i32)
        self.cand_score = torch.empty(self.G, dtype=torch.int64, device=dev)
        self.grant_job = torch.empty(self.G, **i32)
        self.grant_cut = torch.empty(self.G, **i32)
        self.grant_score = torch.empty(self.G, dtype=torch.int64, device=dev)
        self.job_gap = torch.empty(self.J, **i32)
        self.rounds = torch.zeros(2, **i32)
        self.metrics = torch.zeros(4, dtype=torch.int64, device=dev)
        engine.ensure_workspace(self.G, self.J, self.S)

    def prepare(self):
        self.engine.sja_prepare_profiles(self.seg_off, self.dur, self.mem, self.safe, self.progress,
                                         self.pre_dur, self.pre_peak, self.prev_safe)

    def fit(self):
        self.engine.sja_fit(self.W, self.C, self.cut, self.bits)

    def select(self, params: Params, job_held=None, gap_active=None):
        self.engine.sja_select(params, self.wait, self.sla_class, job_held, gap_active,
                               self.cand_job, self.cand_cut, self.cand_score)

    def fit_select(self, params: Params, job_held=None, gap_active=None):
        self.engine.sja_fit_select(self.W, self.C, params, self.wait, self.sla_class, job_held, gap_active,
                                   self.cand_job, self.cand_cut, self.cand_score)

    def set_gaps(self, W, C):
        """The next tick's gaps (numpy int32, the same count as before), copied into place."""
        self.W.copy_(torch.from_numpy(np.ascontiguousarray(W)))
        self.C.copy_(torch.from_numpy(np.ascontiguousarray(C)))

    def advance(self, wait_step: int):
        self.engine.sja_advance(self.W, self.C, self.grant_job, self.grant_cut, self.job_gap,
                                self.progress, self.wait, wait_step, self.metrics)

    def resolve(self, params: Params):
        self.engine.sja_resolve(params, self.wait, self.sla_class, self.grant_job, self.grant_cut,
                                self.grant_score, self.job_gap, self.rounds)
