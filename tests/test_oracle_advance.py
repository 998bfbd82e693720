"""Pins for the CPU oracle's tick advance (no GPU).

A parent job resumes from its last completed fragment (Sec. 3.1, 3.5), so a
grant moves the job's progress point to the granted safe boundary.  Checked
against a pure-Python restatement that works on the raw segments, and against
what must hold over a chain of ticks: progress only grows, stays on safe
boundaries and inside the job; the filled area never exceeds the offered area
because every grant fits its gap by construction (Sec. 3.4); with roomy gaps
every job completes.
"""
import numpy as np
import pytest

from gen import make_gaps, make_workload
from oracle import brute
from helpers import random_gaps, random_jobs, random_prefs


def _tick(O, seg_off, dur, mem, safe, progress, W, C, par, wait, cls):
    pd, pp, _ = O.prepare(seg_off, dur, mem, safe, progress)
    cut, _ = O.fit(seg_off, dur, mem, safe, progress, W, C, False)
    gj, gc, gs, jg, rounds, stable = O.resolve(cut, seg_off, pd, pp, par, wait, cls)
    assert stable
    return pd, pp, gj, gc, jg


@pytest.mark.parametrize("policy", [0, 1, 2, 3])
def test_advance_matches_raw_segment_brute_force(oracle, policy):
    rng = np.random.default_rng(700 + policy)
    for case in range(150):
        n_jobs, n_gaps = int(rng.integers(1, 8)), int(rng.integers(1, 6))
        seg_off, dur, mem, safe, progress = random_jobs(rng, n_jobs, 0, 9, d_hi=4, m_hi=4)
        W, C = random_gaps(rng, n_gaps, 25, 5)
        wait, cls = random_prefs(rng, n_jobs, wait_hi=9)
        if case % 5 == 0:
            wait[rng.integers(0, n_jobs)] = 2**31 - 2          # saturates, never wraps
        par = oracle.Params.make(policy, wait_scale=1, sla_weight=(3, 2, 1))
        if case % 5 == 0:
            par = oracle.Params.make(0)
        pd, pp, gj, gc, jg = _tick(oracle, seg_off, dur, mem, safe, progress, W, C, par, wait, cls)
        step = int(rng.integers(0, 4))
        p2, w2, m = oracle.advance(seg_off, pd, pp, W, C, gj, gc, jg, progress, wait, step)
        bp, bw, bm = brute.advance(seg_off, dur, mem, W, C, gj, gc, progress, wait, step)
        assert p2.tolist() == bp
        assert w2.tolist() == bw
        assert m.tolist() == bm


def test_advance_leaves_inputs_alone_and_wait_is_optional(oracle):
    rng = np.random.default_rng(3)
    seg_off, dur, mem, safe, progress = random_jobs(rng, 6, 1, 8)
    W, C = random_gaps(rng, 4, 30, 9)
    wait, cls = random_prefs(rng, 6)
    par = oracle.Params.make(0)
    pd, pp, gj, gc, jg = _tick(oracle, seg_off, dur, mem, safe, progress, W, C, par, wait, cls)
    p0, w0 = progress.copy(), wait.copy()
    p2, w2, m = oracle.advance(seg_off, pd, pp, W, C, gj, gc, jg, progress, None, 5)
    assert w2 is None and (progress == p0).all() and (wait == w0).all()
    p3, _, m3 = oracle.advance(seg_off, pd, pp, W, C, gj, gc, jg, progress, wait, 5)
    assert (p2 == p3).all() and (m == m3).all()


def test_no_grants_means_only_waiting(oracle):
    rng = np.random.default_rng(4)
    seg_off, dur, mem, safe, progress = random_jobs(rng, 9, 0, 6)
    lens = np.diff(seg_off)
    W = np.array([0, 5], dtype=np.int32)
    C = np.array([7, 0], dtype=np.int32)                      # nothing fits a flat gap
    wait = np.arange(9, dtype=np.int32)
    pd, pp, _ = oracle.prepare(seg_off, dur, mem, safe, progress)
    none_g = np.full(2, -1, dtype=np.int32)
    none_j = np.full(9, -1, dtype=np.int32)
    p2, w2, m = oracle.advance(seg_off, pd, pp, W, C, none_g, none_g, none_j, progress, wait, 3)
    assert (p2 == progress).all()
    assert (w2 == np.where(progress < lens, wait + 3, wait)).all()
    assert m.tolist() == [0, 0, 0, int((progress >= lens).sum())]


def test_inconsistent_grant_tables_are_rejected(oracle):
    seg_off = np.array([0, 3, 5], dtype=np.int64)
    dur = np.ones(5, dtype=np.int32)
    mem = np.ones(5, dtype=np.int32)
    safe = np.ones(5, dtype=np.uint8)
    progress = np.array([1, 0], dtype=np.int32)
    pd, pp, _ = oracle.prepare(seg_off, dur, mem, safe, progress)
    W = np.array([9], dtype=np.int32)
    C = np.array([9], dtype=np.int32)
    i32 = lambda *v: np.array(v, dtype=np.int32)              # noqa: E731
    ok = oracle.advance(seg_off, pd, pp, W, C, i32(0), i32(3), i32(0, -1), progress, None, 1)
    assert ok[0].tolist() == [3, 0] and ok[2].tolist() == [2 * 1, 81, 1, 1]
    with pytest.raises(Exception):                            # job table does not point back
        oracle.advance(seg_off, pd, pp, W, C, i32(0), i32(3), i32(-1, -1), progress, None, 1)
    with pytest.raises(Exception):                            # cut does not move the job forward
        oracle.advance(seg_off, pd, pp, W, C, i32(0), i32(1), i32(0, -1), progress, None, 1)
    with pytest.raises(Exception):                            # cut beyond the job's end
        oracle.advance(seg_off, pd, pp, W, C, i32(0), i32(4), i32(0, -1), progress, None, 1)
    with pytest.raises(Exception):                            # job claims a gap that went elsewhere
        oracle.advance(seg_off, pd, pp, W, C, i32(0), i32(3), i32(0, 0), progress, None, 1)


@pytest.mark.parametrize("policy", [0, 3])
def test_chain_of_ticks_invariants(oracle, policy):
    w = make_workload("small", 5, n_gaps=48, n_jobs=300)
    lens = np.diff(w.seg_off)
    par = oracle.Params.make(policy)
    progress, wait = w.progress.copy(), w.wait.copy()
    total_filled = 0
    for tick in range(6):
        W, C = (w.W, w.C) if tick == 0 else make_gaps("small", 5, tick, 48)
        pd, pp, gj, gc, jg = _tick(oracle, w.seg_off, w.dur, w.mem, w.safe, progress, W, C, par,
                                   wait, w.sla_class)
        p2, w2, m = oracle.advance(w.seg_off, pd, pp, W, C, gj, gc, jg, progress, wait, 1000)
        moved = p2 != progress
        assert (p2 >= progress).all() and (p2 <= lens).all()
        assert (moved == (jg >= 0)).all()
        assert w.safe[w.seg_off[:-1][moved] + p2[moved] - 1].all()       # lands on safe boundaries
        assert (w2[moved] == 0).all()
        still = ~moved & (progress < lens)
        assert (w2[still] == np.minimum(wait[still].astype(np.int64) + 1000, 2**31 - 1)).all()
        assert 0 < m[0] <= m[1] and m[2] == moved.sum() <= 48
        assert m[3] == (p2 >= lens).sum()
        total_filled += int(m[0])
        progress, wait = p2, w2
    assert total_filled > 0


def test_roomy_gaps_complete_every_job(oracle):
    rng = np.random.default_rng(11)
    seg_off, dur, mem, safe, progress = random_jobs(rng, 12, 1, 9, allow_done=False)
    safe[seg_off[1:] - 1] = 1
    progress[:] = 0
    wait, cls = random_prefs(rng, 12)
    W = np.full(3, 1000, dtype=np.int32)
    C = np.full(3, 1000, dtype=np.int32)
    par = oracle.Params.make(1)
    lens = np.diff(seg_off)
    work = int(sum(int(dur[seg_off[j]:seg_off[j + 1]].sum()) * int(mem[seg_off[j]:seg_off[j + 1]].max())
                   for j in range(12)))
    filled = 0
    for tick in range(4):                                      # 3 whole jobs per tick
        pd, pp, gj, gc, jg = _tick(oracle, seg_off, dur, mem, safe, progress, W, C, par, wait, cls)
        progress, wait, m = oracle.advance(seg_off, pd, pp, W, C, gj, gc, jg, progress, wait, 1)
        filled += int(m[0])
        assert m[2] == 3 and m[3] == 3 * (tick + 1)
    assert (progress == lens).all()
    assert filled == work                                      # whole jobs: duration x peak of each
