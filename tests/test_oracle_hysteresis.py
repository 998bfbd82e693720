"""Pins for the oracle's hysteresis fit (no GPU).

Sec. 3.9 names the rule (a minimum gain in slack before a further subdivision is
accepted) without a formula; the oracle's header states the reading.  Pinned by a
hand-worked example (tests/golden/hysteresis_worked_example.json), a brute force
that builds the set of admitted boundaries from scratch, reductions to the plain
and the limited fit, and properties that hold for every pair.
"""
import json
import os

import numpy as np
import pytest

from oracle import brute
from helpers import random_gaps, random_jobs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hysteresis_worked_example.json")


def _case(rng, n_jobs=5, n_gaps=5):
    seg_off, dur, mem, safe, progress = random_jobs(rng, n_jobs, 0, 12, d_hi=4, m_hi=9, safe_p=0.6)
    power = rng.integers(0, 7, size=len(dur)).astype(np.int32)
    W, C = random_gaps(rng, n_gaps, 45, 12)
    deadline = rng.integers(-3, 40, size=n_jobs).astype(np.int32)
    n_caps = int(rng.integers(2, 6))
    cap_set = np.sort(rng.choice(np.arange(0, 12), size=n_caps, replace=False)).astype(np.int32)
    return seg_off, dur, mem, safe, progress, power, W, C, deadline, cap_set


def test_worked_example(oracle):
    with open(GOLDEN) as f:
        ex = json.load(f)
    dur = np.array(ex["dur_s"], dtype=np.int32)
    mem = np.array(ex["mem_gb"], dtype=np.int32)
    safe = np.array(ex["safe"], dtype=np.uint8)
    seg_off = np.array([0, len(dur)], dtype=np.int64)
    progress = np.zeros(1, dtype=np.int32)
    for case in ex["cases"]:
        W = np.array([case["W"]], dtype=np.int32)
        C = np.array([case["C"]], dtype=np.int32)
        cut, bits = oracle.fit_hysteresis(seg_off, dur, mem, safe, progress, W, C, case["cap_set"],
                                          case["min_gain"], want_bits=True)
        assert int(cut[0, 0]) == case["expected_cut"], case
        assert int(bits[0, 0]) == (1 if case["expected_cut"] >= 0 else 0)
        assert brute.fit_one_hysteresis(list(dur), list(mem), list(safe), 0, case["W"], case["C"],
                                        case["cap_set"], case["min_gain"]) == case["expected_cut"], case


def test_matches_the_set_definition_brute_force(oracle):
    rng = np.random.default_rng(31)
    moved = 0
    for case in range(300):
        seg_off, dur, mem, safe, progress, power, W, C, deadline, cap_set = _case(rng)
        min_gain = int(rng.integers(1, 5))
        with_limits = case % 2 == 1
        tau_min, tau_max = int(rng.integers(0, 9)), int(rng.integers(4, 30))
        cap, now = int(rng.integers(2, 7)), int(rng.integers(0, 12))
        use_pow, use_dl = with_limits and case % 4 == 1, with_limits and case % 3 != 0
        lim = oracle.Limits.make(tau_min, tau_max, cap, now) if with_limits else None
        cut, bits = oracle.fit_hysteresis(seg_off, dur, mem, safe, progress, W, C, cap_set, min_gain, lim,
                                          power if use_pow else None, deadline if use_dl else None, True)
        plain, _ = oracle.fit_limited(seg_off, dur, mem, safe, progress, W, C, lim,
                                      power if use_pow else None, deadline if use_dl else None)
        moved += int((cut != plain).sum())
        for g in range(len(W)):
            for j in range(len(progress)):
                sl = lambda a: brute.job_slices(seg_off, a, j)          # noqa: E731
                kw = {}
                if with_limits:
                    kw = dict(tau_min=tau_min, tau_max=tau_max, power=sl(power) if use_pow else None,
                              power_cap=cap, deadline=int(deadline[j]) if use_dl else None, now=now)
                want = brute.fit_one_hysteresis(sl(dur), sl(mem), sl(safe), int(progress[j]), int(W[g]),
                                                int(C[g]), list(cap_set), min_gain, **kw)
                assert int(cut[g, j]) == want, (case, g, j)
                assert bool((bits[g, j >> 5] >> (j & 31)) & 1) == (want >= 0)
    assert moved > 200          # the rule did act


def test_reductions_to_the_fit_without_hysteresis(oracle):
    rng = np.random.default_rng(32)
    for _ in range(60):
        seg_off, dur, mem, safe, progress, power, W, C, deadline, cap_set = _case(rng, 7, 6)
        plain, pbits = oracle.fit(seg_off, dur, mem, safe, progress, W, C, True)
        # no capacity set: the rule is off
        a, abits = oracle.fit_hysteresis(seg_off, dur, mem, safe, progress, W, C, [], 1, want_bits=True)
        assert (a == plain).all() and (abits == pbits).all()
        # one capacity that covers everything: every boundary maps to it, no gain to be had
        b, _ = oracle.fit_hysteresis(seg_off, dur, mem, safe, progress, W, C, [100], 1)
        assert (b == plain).all()
        # a gain larger than the whole range of a set that covers everything
        c, _ = oracle.fit_hysteresis(seg_off, dur, mem, safe, progress, W, C, [0, 3, 6, 50], 51)
        assert (c == plain).all()
        # limits pass through
        lim = oracle.Limits.make(2, 20, 5, 3)
        want, _ = oracle.fit_limited(seg_off, dur, mem, safe, progress, W, C, lim, power, deadline)
        d, _ = oracle.fit_hysteresis(seg_off, dur, mem, safe, progress, W, C, [], 1, lim, power, deadline)
        assert (d == want).all()


def test_properties_of_every_pair(oracle):
    rng = np.random.default_rng(33)
    for _ in range(80):
        seg_off, dur, mem, safe, progress, power, W, C, deadline, cap_set = _case(rng, 7, 6)
        min_gain = int(rng.integers(1, 6))
        plain, _ = oracle.fit(seg_off, dur, mem, safe, progress, W, C, False)
        got, _ = oracle.fit_hysteresis(seg_off, dur, mem, safe, progress, W, C, cap_set, min_gain)
        _, pp, _ = oracle.prepare(seg_off, dur, mem, safe, progress)
        assert ((got >= 0) == (plain >= 0)).all()              # interest is untouched
        assert (got <= plain).all()                            # never a longer fragment
        G, J = got.shape
        for g in range(G):
            for j in range(J):
                h, s = int(got[g, j]), int(plain[g, j])
                if h == s:
                    continue
                assert safe[seg_off[j] + h - 1]                 # still a checkpoint
                cov_h = brute.cover_one(int(pp[seg_off[j] + h - 1]), cap_set)
                cov_s = brute.cover_one(int(pp[seg_off[j] + s - 1]), cap_set)
                assert cov_h is not None
                assert cov_s is None or cov_s - cov_h >= min_gain       # the gain was there


def test_pairs_agree_with_the_matrix(oracle):
    rng = np.random.default_rng(34)
    for _ in range(20):
        seg_off, dur, mem, safe, progress, power, W, C, deadline, cap_set = _case(rng, 9, 7)
        lim = oracle.Limits.make(1, 25, 5, 2)
        cut, _ = oracle.fit_hysteresis(seg_off, dur, mem, safe, progress, W, C, cap_set, 2, lim, power, deadline)
        G, J = cut.shape
        gi = np.repeat(np.arange(G, dtype=np.int32), J)
        ji = np.tile(np.arange(J, dtype=np.int32), G)
        pc, sd, sp = oracle.fit_pairs_hysteresis(gi, ji, seg_off, dur, mem, safe, progress, W, C, cap_set, 2,
                                                 lim, power, deadline)
        assert (pc.reshape(G, J) == cut).all()
        pd, pp, _ = oracle.prepare(seg_off, dur, mem, safe, progress)
        for i in np.flatnonzero(pc >= 0):
            k = seg_off[ji[i]] + pc[i] - 1
            assert sd[i] == pd[k] and sp[i] == pp[k]


def test_bad_arguments_are_rejected(oracle):
    rng = np.random.default_rng(1)
    seg_off, dur, mem, safe, progress, power, W, C, deadline, cap_set = _case(rng)
    with pytest.raises(Exception):
        oracle.fit_hysteresis(seg_off, dur, mem, safe, progress, W, C, [1, 2], 0)        # min_gain < 1
    with pytest.raises(Exception):
        oracle.fit_hysteresis(seg_off, dur, mem, safe, progress, W, C, [3, 2], 1)        # not ascending
