"""Seeded synthetic workloads for one scheduling tick.

A workload is what the scheduler holds when it advertises a batch of execution
gaps (Sec. 3.5: an offer is a time interval plus a slice capacity) to a set of
waiting jobs, each described by a memory-over-time profile (Sec. 3.2-3.3) that
is already the risk-adjusted envelope U(t) of Sec. 3.9, cut into
piecewise-constant segments with flagged subjob boundaries (Sec. 3.7).

Array conventions (all numpy, C-contiguous):

  seg_off   int64 [J+1]  CSR offsets; job j owns segments seg_off[j]..seg_off[j+1]-1
  dur       int32 [S]    segment duration in ticks, >= 1
  mem       int32 [S]    segment memory in MiB
  safe      uint8 [S]    entry k of a job = flag of boundary k+1 (boundary b lies
                         before segment b; boundary L is the job's end, flag 1)
  progress  int32 [J]    boundary index the job has completed up to, 0 <= p < L
  W, C      int32 [G]    gap window (ticks) and capacity (MiB)
  wait      int32 [J]    waiting time carried as a preference
  sla_class uint8 [J]    0 (most urgent), 1, 2

Draw order, fixed so that a (config, seed) pair always yields the same arrays:
lengths, durations, memory, safe flags, progress, W, C, wait, class -- each as
one vectorised draw over all jobs / segments / gaps from a single
numpy.random.Generator(PCG64(seed)).  The only floating point in the
repository lives here (log-uniform and Pareto transforms).
"""
from __future__ import annotations

import dataclasses
import zlib
from typing import Dict, Optional, Sequence, Tuple, Union

import numpy as np

POLICY_EFFICIENCY = 0
POLICY_FAIRNESS = 1
POLICY_SLA = 2
POLICY_MIXED = 3


@dataclasses.dataclass(frozen=True)
class Config:
    """Recipe for one named workload."""

    name: str
    n_gaps: int
    n_jobs: int
    seg_len: Union[int, Tuple[int, int]]          # fixed L, or (lo, hi) inclusive
    dur: Tuple = ("uniform", 1, 100)              # or ("pareto", alpha, lo, hi)
    mem: Tuple = ("loguniform", 256, 40960)       # or ("bimodal", ...), ("walk", lo, hi)
    safe_p: float = 0.25
    w_range: Tuple[int, int] = (50, 2000)
    c_set: Sequence[int] = (5120, 10240, 20480, 40960)
    policy: int = POLICY_EFFICIENCY
    max_rounds: int = 0                           # 0 = until stable


CONFIGS: Dict[str, Config] = {
    "tiny": Config("tiny", 8, 16, 64),
    "small": Config("small", 256, 1024, 256, policy=POLICY_FAIRNESS),
    "medium": Config(
        "medium", 2048, 8192, 512,
        mem=("bimodal", 0.7, (256, 8192), (16384, 81920)),
        w_range=(100, 20000),
        c_set=(9216, 18432, 36864, 73728, 147456),
        policy=POLICY_SLA,
    ),
    "large": Config(
        "large", 8192, 32768, 1024,
        dur=("pareto", 1.5, 1, 100000),
        safe_p=0.1,
        policy=POLICY_EFFICIENCY,
        max_rounds=8,
    ),
    "stress": Config(
        "stress", 32768, 65536, (16, 2048),
        mem=("walk", 256, 147456),
        w_range=(10, 100000),
        c_set=tuple(u * 36864 for u in range(1, 9)),
        policy=POLICY_MIXED,
    ),
}


def config_names():
    return list(CONFIGS)


@dataclasses.dataclass
class Workload:
    name: str
    seed: int
    n_gaps: int
    n_jobs: int
    seg_off: np.ndarray
    dur: np.ndarray
    mem: np.ndarray
    safe: np.ndarray
    progress: np.ndarray
    W: np.ndarray
    C: np.ndarray
    wait: np.ndarray
    sla_class: np.ndarray
    policy: int
    max_rounds: int
    wait_scale: int = 1000
    sla_weight: Tuple[int, int, int] = (4, 2, 1)
    class0_override: int = 1

    @property
    def n_segments(self) -> int:
        return int(self.seg_off[-1])

    def checksums(self) -> Dict[str, int]:
        """CRC32 of every array, for logs and reproducibility checks."""
        out = {}
        for k in ("seg_off", "dur", "mem", "safe", "progress", "W", "C", "wait", "sla_class"):
            out[k] = zlib.crc32(np.ascontiguousarray(getattr(self, k)).tobytes())
        return out


def _loguniform_int(rng: np.random.Generator, lo: int, hi: int, n: int) -> np.ndarray:
    """floor(lo * (hi/lo)**u), u ~ U[0,1), clipped to [lo, hi]."""
    u = rng.random(n)
    v = np.floor(lo * np.power(hi / lo, u))
    return np.clip(v, lo, hi).astype(np.int32)


def _draw_durations(rng, spec, n):
    kind = spec[0]
    if kind == "uniform":
        return rng.integers(spec[1], spec[2] + 1, size=n, dtype=np.int64).astype(np.int32)
    if kind == "pareto":
        _, alpha, lo, hi = spec
        u = rng.random(n)
        v = np.floor(np.power(1.0 - u, -1.0 / alpha))      # scale x_m = 1
        return np.clip(v, lo, hi).astype(np.int32)
    raise ValueError(f"unknown duration spec {spec!r}")


def _draw_memory(rng, spec, seg_off, n):
    kind = spec[0]
    if kind == "loguniform":
        return _loguniform_int(rng, spec[1], spec[2], n)
    if kind == "bimodal":
        _, p_low, (l0, l1), (h0, h1) = spec
        pick = rng.random(n) < p_low
        low = _loguniform_int(rng, l0, l1, n)
        high = _loguniform_int(rng, h0, h1, n)
        return np.where(pick, low, high).astype(np.int32)
    if kind == "walk":
        # m_0 log-uniform; m_{k+1} = clip(m_k + s_k * floor(m_k / 10), lo, hi), s_k = +-1.
        _, lo, hi = spec
        n_jobs = len(seg_off) - 1
        lens = np.diff(seg_off)
        start = _loguniform_int(rng, lo, hi, n_jobs).astype(np.int64)
        sign = (rng.integers(0, 2, size=n, dtype=np.int8) * 2 - 1).astype(np.int8)
        out = np.empty(n, dtype=np.int32)
        l_max = int(lens.max()) if n_jobs else 0
        cur = start.copy()
        for k in range(l_max):
            alive = np.nonzero(lens > k)[0]
            pos = seg_off[alive] + k
            if k > 0:
                prev = cur[alive]
                step = sign[pos - 1].astype(np.int64) * (prev // 10)
                cur[alive] = np.clip(prev + step, lo, hi)
            out[pos] = cur[alive]
        return out
    raise ValueError(f"unknown memory spec {spec!r}")


def _draw_progress(rng, seg_off, safe):
    """Uniform over {0} plus the flagged internal boundaries 1..L-1 of each job."""
    n_jobs = len(seg_off) - 1
    internal = safe.astype(np.int64)
    internal[seg_off[1:] - 1] = 0                      # the end is not a progress point
    cs = np.cumsum(internal)
    before = np.concatenate(([0], cs))[seg_off[:-1]]   # flags counted before each job
    n_int = np.concatenate(([0], cs))[seg_off[1:]] - before
    u = rng.random(n_jobs)
    pick = np.minimum(np.floor(u * (n_int + 1)).astype(np.int64), n_int)
    # pick == 0 -> boundary 0; otherwise the pick-th flagged internal boundary
    seg = np.searchsorted(cs, before + pick, side="left")
    prog = np.where(pick == 0, 0, seg - seg_off[:-1] + 1)
    return prog.astype(np.int32)


def make_workload(name: str, seed: int = 0, *, n_gaps: Optional[int] = None,
                  n_jobs: Optional[int] = None) -> Workload:
    """Build the named workload; n_gaps / n_jobs shrink it (same distributions)."""
    cfg = CONFIGS[name]
    G = cfg.n_gaps if n_gaps is None else int(n_gaps)
    J = cfg.n_jobs if n_jobs is None else int(n_jobs)
    rng = np.random.Generator(np.random.PCG64(seed))

    if isinstance(cfg.seg_len, tuple):
        lens = rng.integers(cfg.seg_len[0], cfg.seg_len[1] + 1, size=J, dtype=np.int64)
    else:
        lens = np.full(J, cfg.seg_len, dtype=np.int64)
    seg_off = np.zeros(J + 1, dtype=np.int64)
    np.cumsum(lens, out=seg_off[1:])
    S = int(seg_off[-1])

    dur = _draw_durations(rng, cfg.dur, S)
    mem = _draw_memory(rng, cfg.mem, seg_off, S)
    safe = (rng.random(S) < cfg.safe_p).astype(np.uint8)
    safe[seg_off[1:] - 1] = 1                          # the job's end is always safe
    progress = _draw_progress(rng, seg_off, safe)

    W = rng.integers(cfg.w_range[0], cfg.w_range[1] + 1, size=G, dtype=np.int64).astype(np.int32)
    c_set = np.asarray(cfg.c_set, dtype=np.int32)
    C = c_set[rng.integers(0, len(c_set), size=G)]
    wait = rng.integers(0, 10**6 + 1, size=J, dtype=np.int64).astype(np.int32)
    sla_class = rng.integers(0, 3, size=J, dtype=np.int64).astype(np.uint8)

    return Workload(
        name=name, seed=seed, n_gaps=G, n_jobs=J,
        seg_off=seg_off, dur=dur, mem=mem, safe=safe, progress=progress,
        W=np.ascontiguousarray(W), C=np.ascontiguousarray(C),
        wait=wait, sla_class=sla_class,
        policy=cfg.policy, max_rounds=cfg.max_rounds,
    )


def make_gaps(name: str, seed: int, tick: int, n_gaps: Optional[int] = None):
    """The gaps a scheduler advertises at a later tick of the same workload: a fresh (W, C)
    batch with the config's distributions, from its own stream (seed, tick)."""
    cfg = CONFIGS[name]
    G = cfg.n_gaps if n_gaps is None else int(n_gaps)
    rng = np.random.Generator(np.random.PCG64([int(seed), 1000003 + int(tick)]))
    W = rng.integers(cfg.w_range[0], cfg.w_range[1] + 1, size=G, dtype=np.int64).astype(np.int32)
    c_set = np.asarray(cfg.c_set, dtype=np.int32)
    C = c_set[rng.integers(0, len(c_set), size=G)]
    return np.ascontiguousarray(W), np.ascontiguousarray(C)


def make_channels(wl: Workload, seed: int):
    """A second profile channel and per-job deadlines for a workload (inputs only):
    power [n_segments] int32 in watts, a floor plus a share that follows the segment's memory
    with multiplicative noise (100..~1100 W); deadline [n_jobs] int32, log-uniform between
    1 % and 400 % of the config's widest window, measured from time 0, so that for some jobs
    the deadline is tighter than most windows and for others it never binds."""
    cfg = CONFIGS[wl.name]
    rng = np.random.Generator(np.random.PCG64([int(seed), 2000003]))
    S, J = wl.n_segments, wl.n_jobs
    share = wl.mem.astype(np.float64) / 147456.0
    power = 100.0 + 900.0 * np.clip(share * rng.uniform(0.5, 1.5, size=S), 0.0, 1.1)
    w_hi = float(cfg.w_range[1])
    deadline = np.floor(0.01 * w_hi * (400.0 ** rng.random(J))).astype(np.int64)
    return (np.ascontiguousarray(power.astype(np.int32)),
            np.ascontiguousarray(np.clip(deadline, 0, 2**31 - 1).astype(np.int32)))
