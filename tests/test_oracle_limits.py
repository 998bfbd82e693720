"""Pins for the oracle's admission limits and covering-capacity mapping (no GPU).

Limits: a power trace under a cap and a per-job deadline (Sec. 4.4), minimum and
maximum subjob duration (Sec. 4.3).  Checked against a brute force that tests
every boundary from scratch, and against reductions to the plain fit: an upper
bound on the duration is a narrower window; a deadline is a narrower window per
job; the power test is the memory test on the other channel; a lower bound on
the duration can only turn an answer into a decline.  Covering capacity
(Sec. 3.9): against a set-based restatement.
"""
import numpy as np
import pytest

from oracle import brute
from helpers import random_gaps, random_jobs


def _case(rng, n_jobs=5, n_gaps=5):
    seg_off, dur, mem, safe, progress = random_jobs(rng, n_jobs, 0, 10, d_hi=4, m_hi=5)
    power = rng.integers(0, 7, size=len(dur)).astype(np.int32)
    W, C = random_gaps(rng, n_gaps, 28, 6)
    deadline = rng.integers(-3, 40, size=n_jobs).astype(np.int32)
    return seg_off, dur, mem, safe, progress, power, W, C, deadline


def test_limited_fit_matches_every_boundary_brute_force(oracle):
    rng = np.random.default_rng(2024)
    for case in range(300):
        seg_off, dur, mem, safe, progress, power, W, C, deadline = _case(rng)
        tau_min, tau_max = int(rng.integers(0, 9)), int(rng.integers(0, 30))
        cap, now = int(rng.integers(0, 7)), int(rng.integers(0, 12))
        use_pow, use_dl = case % 2 == 0, case % 3 != 0
        lim = oracle.Limits.make(tau_min, tau_max, cap, now)
        cut, bits = oracle.fit_limited(seg_off, dur, mem, safe, progress, W, C, lim,
                                       power if use_pow else None, deadline if use_dl else None, True)
        for g in range(len(W)):
            for j in range(len(progress)):
                sl = lambda a: brute.job_slices(seg_off, a, j)          # noqa: E731
                want = brute.fit_one_limited(sl(dur), sl(mem), sl(safe), int(progress[j]), int(W[g]),
                                             int(C[g]), tau_min, tau_max, sl(power) if use_pow else None,
                                             cap, int(deadline[j]) if use_dl else None, now)
                assert int(cut[g, j]) == want, (case, g, j)
                assert bool((bits[g, j >> 5] >> (j & 31)) & 1) == (want >= 0)


def test_no_limits_is_the_plain_fit(oracle):
    rng = np.random.default_rng(7)
    for _ in range(40):
        seg_off, dur, mem, safe, progress, power, W, C, deadline = _case(rng, 8, 6)
        plain, _ = oracle.fit(seg_off, dur, mem, safe, progress, W, C, False)
        a, _ = oracle.fit_limited(seg_off, dur, mem, safe, progress, W, C, None)
        b, _ = oracle.fit_limited(seg_off, dur, mem, safe, progress, W, C, oracle.Limits.make())
        big = np.full(len(progress), 2**31 - 1, dtype=np.int32)
        c, _ = oracle.fit_limited(seg_off, dur, mem, safe, progress, W, C, oracle.Limits.make(), power, big)
        assert (a == plain).all() and (b == plain).all() and (c == plain).all()


def test_upper_bounds_are_narrower_windows(oracle):
    rng = np.random.default_rng(8)
    for _ in range(60):
        seg_off, dur, mem, safe, progress, power, W, C, deadline = _case(rng, 7, 6)
        tau_max, now = int(rng.integers(0, 25)), int(rng.integers(0, 9))
        got, _ = oracle.fit_limited(seg_off, dur, mem, safe, progress, W, C,
                                    oracle.Limits.make(tau_max=tau_max))
        want, _ = oracle.fit(seg_off, dur, mem, safe, progress, np.minimum(W, tau_max).astype(np.int32), C, False)
        assert (got == want).all()
        got, _ = oracle.fit_limited(seg_off, dur, mem, safe, progress, W, C,
                                    oracle.Limits.make(now=now), None, deadline)
        for j in range(len(progress)):                                    # one job at a time: its own window
            Wj = np.minimum(W.astype(np.int64), int(deadline[j]) - now).astype(np.int32)
            col, _ = oracle.fit(seg_off, dur, mem, safe, progress, Wj, C, False)
            assert (got[:, j] == col[:, j]).all()


def test_power_channel_is_the_memory_test_on_the_other_trace(oracle):
    rng = np.random.default_rng(9)
    for _ in range(60):
        seg_off, dur, mem, safe, progress, power, W, C, deadline = _case(rng, 7, 6)
        cap = int(rng.integers(0, 7))
        # memory unconstrained, power capped == the plain fit run on the power trace with C = cap
        roomy = np.full(len(W), 2**30, dtype=np.int32)
        got, _ = oracle.fit_limited(seg_off, dur, mem, safe, progress, W, roomy,
                                    oracle.Limits.make(power_cap=cap), power)
        want, _ = oracle.fit(seg_off, dur, power, safe, progress, W, np.full(len(W), cap, dtype=np.int32), False)
        assert (got == want).all()
        # both channels: the smaller of the two single-channel answers (both walks stop at their first violation)
        both, _ = oracle.fit_limited(seg_off, dur, mem, safe, progress, W, C,
                                     oracle.Limits.make(power_cap=cap), power)
        only_mem, _ = oracle.fit(seg_off, dur, mem, safe, progress, W, C, False)
        assert (both == np.minimum(only_mem, want)).all()


def test_minimum_duration_only_turns_answers_into_declines(oracle):
    rng = np.random.default_rng(10)
    hit = 0
    for _ in range(80):
        seg_off, dur, mem, safe, progress, power, W, C, deadline = _case(rng, 7, 6)
        tau_min = int(rng.integers(1, 12))
        lens = np.diff(seg_off)
        plain, _ = oracle.fit(seg_off, dur, mem, safe, progress, W, C, False)
        pd, _, _ = oracle.prepare(seg_off, dur, mem, safe, progress)
        got, _ = oracle.fit_limited(seg_off, dur, mem, safe, progress, W, C, oracle.Limits.make(tau_min=tau_min))
        for g in range(len(W)):
            for j in range(len(progress)):
                c = int(plain[g, j])
                if c < 0:
                    assert got[g, j] == -1
                    continue
                d = int(pd[seg_off[j] + c - 1])
                keep = d >= tau_min or c == lens[j]
                assert got[g, j] == (c if keep else -1)
                hit += not keep
    assert hit > 20


def test_bad_limits_are_rejected(oracle):
    rng = np.random.default_rng(1)
    seg_off, dur, mem, safe, progress, power, W, C, deadline = _case(rng)
    with pytest.raises(Exception):
        oracle.fit_limited(seg_off, dur, mem, safe, progress, W, C, oracle.Limits.make(tau_min=-1))
    with pytest.raises(Exception):
        oracle.fit_limited(seg_off, dur, mem, safe, progress, W, C, oracle.Limits.make(tau_max=-1))


def test_cover_is_the_smallest_capacity_that_holds_the_peak(oracle):
    rng = np.random.default_rng(12)
    none = 0
    for case in range(80):
        seg_off, dur, mem, safe, progress, power, W, C, deadline = _case(rng, 8, 6)
        pd, pp, _ = oracle.prepare(seg_off, dur, mem, safe, progress)
        cut, _ = oracle.fit(seg_off, dur, mem, safe, progress, W, C, False)
        par = oracle.Params.make(0)
        wait = np.zeros(len(progress), dtype=np.int32)
        cls = np.zeros(len(progress), dtype=np.uint8)
        gj, gc, gs, jg, _, _ = oracle.resolve(cut, seg_off, pd, pp, par, wait, cls)
        cap_set = np.unique(rng.integers(0, 7, size=int(rng.integers(0, 5)))).astype(np.int32)
        cov, slack = oracle.cover(seg_off, pp, C, gj, gc, cap_set)
        for g in range(len(W)):
            if gj[g] < 0:
                assert (cov[g], slack[g]) == (-1, 0)
                continue
            j = int(gj[g])
            peak = max(brute.job_slices(seg_off, mem, j)[int(progress[j]):int(gc[g])])
            want = brute.cover_one(peak, cap_set.tolist())
            if want is None:
                none += 1
                assert (cov[g], slack[g]) == (-1, 0)
            else:
                assert cov[g] == want and slack[g] == C[g] - want
                assert peak <= cov[g]
                if want <= C[g]:
                    assert slack[g] >= 0
    assert none > 0
    with pytest.raises(Exception):                                        # the set must ascend
        oracle.cover(seg_off, pp, C, gj, gc, np.array([3, 2], dtype=np.int32))
