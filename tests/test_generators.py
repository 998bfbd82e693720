"""The seeded input generators (inputs only, no method arithmetic): same seed, same arrays; the
documented shapes, ranges and structure of every config (no GPU)."""
import numpy as np
import pytest

from gen import CONFIGS, make_channels, make_gaps, make_workload


@pytest.mark.parametrize("name", ["tiny", "small", "medium"])
def test_same_seed_same_workload(name):
    a, b, c = make_workload(name, 3), make_workload(name, 3), make_workload(name, 4)
    for f in ("seg_off", "dur", "mem", "safe", "progress", "W", "C", "wait", "sla_class"):
        np.testing.assert_array_equal(getattr(a, f), getattr(b, f))
    assert any((getattr(a, f) != getattr(c, f)).any() for f in ("dur", "mem", "W"))


@pytest.mark.parametrize("name", ["tiny", "small", "medium", "large"])
def test_workload_structure(name):
    cfg = CONFIGS[name]
    wl = make_workload(name, 0)
    lens = np.diff(wl.seg_off)
    assert wl.seg_off[0] == 0 and wl.seg_off[-1] == len(wl.dur) == len(wl.mem) == len(wl.safe)
    assert (lens >= 1).all() and wl.n_jobs == cfg.n_jobs and wl.n_gaps == cfg.n_gaps
    assert wl.dur.dtype == np.int32 and wl.mem.dtype == np.int32 and wl.safe.dtype == np.uint8
    assert (wl.dur >= 1).all() and (wl.mem >= 0).all()
    assert wl.safe[wl.seg_off[1:] - 1].all()                            # a job's end is a safe boundary
    assert ((wl.progress >= 0) & (wl.progress < lens)).all()            # every job has work left
    at = wl.progress > 0
    assert wl.safe[wl.seg_off[:-1][at] + wl.progress[at] - 1].all()     # progress stands on a safe boundary
    assert (wl.W >= cfg.w_range[0]).all() and (wl.W <= cfg.w_range[1]).all()
    assert set(np.unique(wl.C).tolist()) <= set(cfg.c_set)
    assert (wl.sla_class <= 2).all() and (wl.wait >= 0).all()
    sums = np.add.reduceat(wl.dur.astype(np.int64), wl.seg_off[:-1])
    assert sums.max() <= 2**31 - 1                                      # the int32 precondition of the engine


def test_later_gaps_and_channels_are_seeded_streams_of_their_own():
    wl = make_workload("small", 2)
    W1, C1 = make_gaps("small", 2, 1)
    W1b, C1b = make_gaps("small", 2, 1)
    W2, _ = make_gaps("small", 2, 2)
    np.testing.assert_array_equal(W1, W1b); np.testing.assert_array_equal(C1, C1b)
    assert (W1 != W2).any() and (W1 != wl.W).any() and len(W1) == wl.n_gaps
    assert len(make_gaps("small", 2, 1, 17)[0]) == 17
    cfg = CONFIGS["small"]
    assert (W1 >= cfg.w_range[0]).all() and (W1 <= cfg.w_range[1]).all() and set(np.unique(C1)) <= set(cfg.c_set)
    p, d = make_channels(wl, 2)
    p2, d2 = make_channels(wl, 2)
    np.testing.assert_array_equal(p, p2); np.testing.assert_array_equal(d, d2)
    assert p.dtype == np.int32 and d.dtype == np.int32 and len(p) == wl.n_segments and len(d) == wl.n_jobs
    assert p.min() >= 100 and p.max() <= 1100 and (d >= 0).all()
    assert (d < cfg.w_range[1]).mean() > 0.3 and (d > cfg.w_range[1]).mean() > 0.1   # some bind, some never do
