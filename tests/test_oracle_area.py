"""Pins for the oracle's area-under-the-envelope score (no GPU): the alternative reading of
"filled capacity-time", F = sum of dur * mem over the subjob instead of duration x peak.
Checked against numpy's cumulative sum, a brute force that recomputes every key from the raw
segments and sorts, and two reductions: on flat memory profiles the area is the rectangle, and
the area never exceeds it."""
import numpy as np
import pytest

from gen import make_workload
from oracle import brute
from helpers import random_gaps, random_jobs, random_prefs


@pytest.mark.parametrize("name", ["tiny", "small"])
def test_area_is_a_cumulative_sum_from_the_progress_point(oracle, name):
    wl = make_workload(name, 1)
    a = oracle.area(wl.seg_off, wl.dur, wl.mem, wl.progress)
    pd, pp, _ = oracle.prepare(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress)
    for j in range(wl.n_jobs):
        b, e, p = int(wl.seg_off[j]), int(wl.seg_off[j + 1]), int(wl.progress[j])
        want = np.cumsum(wl.dur[b + p:e].astype(np.int64) * wl.mem[b + p:e].astype(np.int64))
        np.testing.assert_array_equal(a[b + p:e], want)
        assert (a[b:b + p] == -7).all()                                  # before the progress point: untouched
        assert (a[b + p:e] <= pd[b + p:e] * pp[b + p:e]).all()           # never more than the rectangle


@pytest.mark.parametrize("policy", [0, 1, 2, 3])
def test_area_select_and_resolve_match_brute_force(oracle, policy):
    rng = np.random.default_rng(900 + policy)
    differs = 0
    for case in range(120):
        n_jobs, n_gaps = int(rng.integers(1, 7)), int(rng.integers(1, 6))
        seg_off, dur, mem, safe, progress = random_jobs(rng, n_jobs, 0, 10, d_hi=4, m_hi=4)
        W, C = random_gaps(rng, n_gaps, 30, 5)
        wait, cls = random_prefs(rng, n_jobs, wait_hi=3)
        pd, pp, _ = oracle.prepare(seg_off, dur, mem, safe, progress)
        pa = oracle.area(seg_off, dur, mem, progress)
        cut, _ = oracle.fit(seg_off, dur, mem, safe, progress, W, C, False)
        par = oracle.Params.make(policy, wait_scale=2, sla_weight=(3, 2, 1))
        cj, cc, cs = oracle.select(cut, seg_off, pd, pp, par, wait, cls, pre_area=pa)
        rj, rc_, rs = oracle.select(cut, seg_off, pd, pp, par, wait, cls)
        differs += int((cj != rj).any() or (cs != rs).any())
        for g in range(n_gaps):
            want = brute.select_gap(cut[g].tolist(), seg_off, dur, mem, progress, wait, cls, policy, 2, (3, 2, 1), 1,
                                    None, True)
            assert (int(cj[g]), int(cc[g]), int(cs[g])) == want
        got = oracle.resolve(cut, seg_off, pd, pp, par, wait, cls, pre_area=pa)
        want = brute.resolve(cut.tolist(), seg_off, dur, mem, progress, wait, cls, policy, 0, 2, (3, 2, 1), 1, True)
        assert [x.tolist() for x in got[:4]] == [list(x) for x in want[:4]]
        assert (got[4], got[5]) == (want[4], want[5])
    assert differs > 10                                                  # the two readings do rank differently


def test_flat_memory_makes_the_area_the_rectangle(oracle):
    wl = make_workload("small", 4, n_gaps=40, n_jobs=200)
    lens = np.diff(wl.seg_off)
    wl.mem[:] = np.repeat(wl.mem[wl.seg_off[:-1]], lens)                 # one memory level per job
    pd, pp, _ = oracle.prepare(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress)
    pa = oracle.area(wl.seg_off, wl.dur, wl.mem, wl.progress)
    cut, _ = oracle.fit(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, wl.W, wl.C, False)
    for policy in range(4):
        par = oracle.Params.make(policy)
        a = oracle.resolve(cut, wl.seg_off, pd, pp, par, wl.wait, wl.sla_class, pre_area=pa)
        b = oracle.resolve(cut, wl.seg_off, pd, pp, par, wl.wait, wl.sla_class)
        for x, y in zip(a, b):
            np.testing.assert_array_equal(x, y)
