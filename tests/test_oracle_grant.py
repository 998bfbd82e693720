"""Pins for the CPU oracle's policy scores, select and resolve (no GPU).

Checked against the from-scratch brute force (full sort per gap, explicit-set
round simulation), closed forms, and the grant invariants: one job per slot
and no state before a grant (Sec. 3.5), at most one gap per job because a
job's fragments are sequential (Sec. 3.1, 3.5), every grant fits by
construction (Sec. 3.4).
"""
import numpy as np
import pytest

from gen import make_workload
from oracle import brute
from helpers import random_gaps, random_jobs, random_prefs

POLICIES = [0, 1, 2, 3]


def _tick(O, seg_off, dur, mem, safe, progress, W, C):
    pd, pp, _ = O.prepare(seg_off, dur, mem, safe, progress)
    cut, _ = O.fit(seg_off, dur, mem, safe, progress, W, C, False)
    return pd, pp, cut


@pytest.mark.parametrize("policy", POLICIES)
def test_select_matches_full_sort_brute_force(oracle, policy):
    rng = np.random.default_rng(100 + policy)
    for case in range(120):
        n_jobs, n_gaps = int(rng.integers(1, 7)), int(rng.integers(1, 6))
        seg_off, dur, mem, safe, progress = random_jobs(rng, n_jobs, 0, 10, d_hi=4, m_hi=4)
        W, C = random_gaps(rng, n_gaps, 30, 5)
        wait, cls = random_prefs(rng, n_jobs, wait_hi=3)
        pd, pp, cut = _tick(oracle, seg_off, dur, mem, safe, progress, W, C)
        held = None
        held_arr = None
        if case % 3 == 0:
            held_arr = np.where(rng.random(n_jobs) < 0.3, 5, -1).astype(np.int32)
            held = set(np.nonzero(held_arr >= 0)[0].tolist())
        act = None
        if case % 4 == 0:
            act = (rng.random(n_gaps) < 0.6).astype(np.uint8)
        par = oracle.Params.make(policy, wait_scale=2, sla_weight=(3, 2, 1))
        cj, cc, cs = oracle.select(cut, seg_off, pd, pp, par, wait, cls, held_arr, act)
        for g in range(n_gaps):
            if act is not None and not act[g]:
                want = (-1, -1, 0)
            else:
                want = brute.select_gap(cut[g].tolist(), seg_off, dur, mem, progress, wait, cls,
                                        policy, 2, (3, 2, 1), 1, held)
            assert (int(cj[g]), int(cc[g]), int(cs[g])) == want


def test_scores_are_bounded_by_the_gap_rectangle(oracle):
    w = make_workload("small", 2, n_gaps=64, n_jobs=256)
    pd, pp, cut = _tick(oracle, w.seg_off, w.dur, w.mem, w.safe, w.progress, w.W, w.C)
    par = oracle.Params.make(0)
    cj, cc, cs = oracle.select(cut, w.seg_off, pd, pp, par, w.wait, w.sla_class)
    has = cj >= 0
    assert has.any()
    assert (cs[has] > 0).all()
    assert (cs[has] <= w.W[has].astype(np.int64) * w.C[has].astype(np.int64)).all()
    # fairness score = F * (1000 + wait) of the winning job, with F read off the raw profile
    parf = oracle.Params.make(1)
    fj, fc, fs = oracle.select(cut, w.seg_off, pd, pp, parf, w.wait, w.sla_class)
    for g in np.nonzero(fj >= 0)[0][:40]:
        j, c = int(fj[g]), int(fc[g])
        a, p = int(w.seg_off[j]), int(w.progress[j])
        F = int(w.dur[a + p:a + c].astype(np.int64).sum()) * int(w.mem[a + p:a + c].max())
        assert int(fs[g]) == F * (1000 + int(w.wait[j]))
        assert int(fs[g]) % (1000 + int(w.wait[j])) == 0


def test_policies_collapse_when_preferences_are_equal(oracle):
    w = make_workload("small", 5, n_gaps=48, n_jobs=200)
    pd, pp, cut = _tick(oracle, w.seg_off, w.dur, w.mem, w.safe, w.progress, w.W, w.C)
    same_wait = np.full(w.n_jobs, 777, dtype=np.int32)
    same_cls = np.full(w.n_jobs, 1, dtype=np.uint8)
    eff = oracle.select(cut, w.seg_off, pd, pp, oracle.Params.make(0), same_wait, same_cls)
    fair = oracle.select(cut, w.seg_off, pd, pp, oracle.Params.make(1), same_wait, same_cls)
    sla = oracle.select(cut, w.seg_off, pd, pp, oracle.Params.make(2), same_wait, same_cls)
    mixed = oracle.select(cut, w.seg_off, pd, pp, oracle.Params.make(3), same_wait, same_cls)
    for other in (fair, sla, mixed):
        np.testing.assert_array_equal(eff[0], other[0])
        np.testing.assert_array_equal(eff[1], other[1])
    np.testing.assert_array_equal(fair[2], eff[2] * 1777)
    np.testing.assert_array_equal(sla[2], eff[2] * 2)
    np.testing.assert_array_equal(mixed[2], fair[2])
    # class-0 override: one class-0 job that is interested anywhere wins there
    cls = same_cls.copy()
    j0 = int(np.argmax((cut >= 0).sum(axis=0)))
    cls[j0] = 0
    ov = oracle.select(cut, w.seg_off, pd, pp, oracle.Params.make(2, sla_weight=(1, 50, 50)),
                       same_wait, cls)
    rows = cut[:, j0] >= 0
    assert rows.any() and (ov[0][rows] == j0).all()
    no = oracle.select(cut, w.seg_off, pd, pp,
                       oracle.Params.make(2, sla_weight=(1, 50, 50), class0_override=0),
                       same_wait, cls)
    assert (no[0][rows] != j0).any()


def test_ties_go_to_the_lower_job_id(oracle):
    """Duplicate a job: the twins tie on every key, the lower id must win; permuting
    ids moves winners with their jobs."""
    rng = np.random.default_rng(9)
    seg_off, dur, mem, safe, progress = random_jobs(rng, 6, 3, 10, d_hi=5, m_hi=5,
                                                    allow_done=False)
    # job 6 := copy of job 2
    a, b = int(seg_off[2]), int(seg_off[3])
    seg_off2 = np.append(seg_off, seg_off[-1] + (b - a))
    dur2 = np.concatenate([dur, dur[a:b]])
    mem2 = np.concatenate([mem, mem[a:b]])
    safe2 = np.concatenate([safe, safe[a:b]])
    prog2 = np.append(progress, progress[2]).astype(np.int32)
    wait = np.array([1, 2, 3, 1, 2, 3, 3], dtype=np.int32)
    cls = np.array([0, 1, 2, 0, 1, 2, 2], dtype=np.uint8)
    W, C = random_gaps(rng, 12, 40, 6)
    pd, pp, cut = _tick(oracle, seg_off2, dur2, mem2, safe2, prog2, W, C)
    np.testing.assert_array_equal(cut[:, 2], cut[:, 6])
    for policy in POLICIES:
        cj, _, _ = oracle.select(cut, seg_off2, pd, pp, oracle.Params.make(policy), wait, cls)
        assert (cj != 6).all()
        held = np.full(7, -1, dtype=np.int32)
        held[2] = 0                                       # with the lower twin held, 6 may win
        cj2, _, _ = oracle.select(cut, seg_off2, pd, pp, oracle.Params.make(policy), wait, cls, held)
        np.testing.assert_array_equal(cj2[cj == 2], 6)


def test_permuting_job_ids_permutes_winners(oracle):
    w = make_workload("small", 8, n_gaps=40, n_jobs=96)
    pd, pp, cut = _tick(oracle, w.seg_off, w.dur, w.mem, w.safe, w.progress, w.W, w.C)
    par = oracle.Params.make(1)
    cj, cc, cs = oracle.select(cut, w.seg_off, pd, pp, par, w.wait, w.sla_class)
    rng = np.random.default_rng(1)
    perm = rng.permutation(w.n_jobs)                      # new job i = old job perm[i]
    lens = np.diff(w.seg_off)[perm]
    so = np.zeros(w.n_jobs + 1, dtype=np.int64)
    np.cumsum(lens, out=so[1:])
    idx = np.concatenate([np.arange(w.seg_off[o], w.seg_off[o + 1]) for o in perm])
    pd2, pp2, cut2 = _tick(oracle, so, w.dur[idx], w.mem[idx], w.safe[idx],
                           w.progress[perm], w.W, w.C)
    cj2, cc2, cs2 = oracle.select(cut2, so, pd2, pp2, par, w.wait[perm], w.sla_class[perm])
    np.testing.assert_array_equal(cs2, cs)                # scores never depend on ids
    has = cj >= 0
    # fairness scores with distinct waits almost never tie: winners move with their jobs
    np.testing.assert_array_equal(perm[cj2[has]], cj[has])


# ----------------------------------------------------------------- resolve
@pytest.mark.parametrize("policy", POLICIES)
def test_resolve_matches_explicit_set_simulation(oracle, policy):
    rng = np.random.default_rng(500 + policy)
    for case in range(80):
        n_jobs, n_gaps = int(rng.integers(1, 8)), int(rng.integers(1, 8))
        seg_off, dur, mem, safe, progress = random_jobs(rng, n_jobs, 0, 8, d_hi=3, m_hi=3)
        W, C = random_gaps(rng, n_gaps, 20, 4)
        wait, cls = random_prefs(rng, n_jobs, wait_hi=2)
        cap = int(rng.integers(0, 4))
        pd, pp, cut = _tick(oracle, seg_off, dur, mem, safe, progress, W, C)
        par = oracle.Params.make(policy, wait_scale=3, sla_weight=(3, 2, 1), max_rounds=cap)
        got = oracle.resolve(cut, seg_off, pd, pp, par, wait, cls)
        want = brute.resolve(cut.tolist(), seg_off, dur, mem, progress, wait, cls, policy, cap,
                             3, (3, 2, 1), 1)
        assert got[0].tolist() == want[0]
        assert got[1].tolist() == want[1]
        assert got[2].tolist() == want[2]
        assert got[3].tolist() == want[3]
        assert got[4:] == want[4:]


@pytest.mark.parametrize("name,policy", [("tiny", 0), ("small", 1), ("small", 3)])
def test_resolve_invariants(oracle, name, policy):
    w = make_workload(name, 0) if name == "tiny" else make_workload(name, 0, n_gaps=96, n_jobs=256)
    pd, pp, cut = _tick(oracle, w.seg_off, w.dur, w.mem, w.safe, w.progress, w.W, w.C)
    par = oracle.Params.make(policy)
    gj, gc, gs, jg, rounds, stable = oracle.resolve(cut, w.seg_off, pd, pp, par, w.wait, w.sla_class)
    assert stable == 1 and rounds >= 1
    granted = np.nonzero(gj >= 0)[0]
    assert len(set(gj[granted].tolist())) == len(granted)            # no job twice
    for g in granted:
        j = int(gj[g])
        assert cut[g, j] == gc[g] and gc[g] >= 0                     # an interested pair
        assert jg[j] == g
        a, p = int(w.seg_off[j]), int(w.progress[j])
        assert w.dur[a + p:a + gc[g]].astype(np.int64).sum() <= w.W[g]   # fits by construction
        assert w.mem[a + p:a + gc[g]].max() <= w.C[g]
    held_jobs = np.nonzero(jg >= 0)[0]
    np.testing.assert_array_equal(gj[jg[held_jobs]], held_jobs)      # job_gap inverts grant_job
    # gap 0 receives its round-1 choice
    cj, cc, cs = oracle.select(cut, w.seg_off, pd, pp, par, w.wait, w.sla_class)
    assert gj[0] == cj[0] and gc[0] == cc[0] and gs[0] == cs[0]
    # stable: an ungranted gap has no un-held interested job left
    act = (gj < 0).astype(np.uint8)
    rj, _, _ = oracle.select(cut, w.seg_off, pd, pp, par, w.wait, w.sla_class, jg, act)
    assert (rj == -1).all()


def test_resolve_closed_form_identical_gaps(oracle):
    """G identical gaps, strictly ranked jobs: gap i gets the (i+1)-th best job in round
    i+1; with a cap of R rounds only gaps 0..R-1 are granted."""
    J, G = 9, 6
    seg_off = np.arange(J + 1, dtype=np.int64)
    dur = np.arange(1, J + 1, dtype=np.int32)              # F = dur * 1, strictly increasing
    mem = np.ones(J, dtype=np.int32)
    safe = np.ones(J, dtype=np.uint8)
    progress = np.zeros(J, dtype=np.int32)
    W = np.full(G, 100, dtype=np.int32)
    C = np.full(G, 5, dtype=np.int32)
    wait = np.zeros(J, dtype=np.int32)
    cls = np.zeros(J, dtype=np.uint8)
    pd, pp, cut = _tick(oracle, seg_off, dur, mem, safe, progress, W, C)
    gj, gc, gs, jg, rounds, stable = oracle.resolve(cut, seg_off, pd, pp, oracle.Params.make(0), wait, cls)
    assert gj.tolist() == [8, 7, 6, 5, 4, 3] and rounds == G and stable == 1
    assert gs.tolist() == [9, 8, 7, 6, 5, 4]
    R = 4
    gj, gc, gs, jg, rounds, stable = oracle.resolve(cut, seg_off, pd, pp,
                                                    oracle.Params.make(0, max_rounds=R), wait, cls)
    assert gj.tolist() == [8, 7, 6, 5, -1, -1] and rounds == R and stable == 0
    assert jg.tolist() == [-1, -1, -1, -1, -1, 3, 2, 1, 0]


def test_resolve_with_distinct_top_choices_is_one_round(oracle):
    """Each gap can only host 'its own' job: one round, grant == select."""
    J = G = 5
    seg_off = np.arange(J + 1, dtype=np.int64)
    dur = np.array([10, 20, 30, 40, 50], dtype=np.int32)
    mem = np.array([5, 4, 3, 2, 1], dtype=np.int32)
    safe = np.ones(J, dtype=np.uint8)
    progress = np.zeros(J, dtype=np.int32)
    # gap g: window fits jobs <= g in duration, capacity fits jobs >= g in memory -> only job g
    W = dur.copy()
    C = mem.copy()
    wait = np.zeros(J, dtype=np.int32)
    cls = np.zeros(J, dtype=np.uint8)
    pd, pp, cut = _tick(oracle, seg_off, dur, mem, safe, progress, W, C)
    assert ((cut >= 0) == np.eye(J, dtype=bool)).all()
    par = oracle.Params.make(0)
    cj, cc, cs = oracle.select(cut, seg_off, pd, pp, par, wait, cls)
    gj, gc, gs, jg, rounds, stable = oracle.resolve(cut, seg_off, pd, pp, par, wait, cls)
    np.testing.assert_array_equal(gj, cj)
    np.testing.assert_array_equal(gc, cc)
    np.testing.assert_array_equal(gs, cs)
    assert rounds == 1 and stable == 1 and jg.tolist() == [0, 1, 2, 3, 4]


def test_resolve_with_no_interest_at_all(oracle):
    seg_off = np.array([0, 2, 4], dtype=np.int64)
    dur = np.array([5, 5, 5, 5], dtype=np.int32)
    mem = np.array([9, 9, 9, 9], dtype=np.int32)
    safe = np.ones(4, dtype=np.uint8)
    progress = np.zeros(2, dtype=np.int32)
    W = np.array([1, 100], dtype=np.int32)
    C = np.array([100, 1], dtype=np.int32)
    pd, pp, cut = _tick(oracle, seg_off, dur, mem, safe, progress, W, C)
    gj, gc, gs, jg, rounds, stable = oracle.resolve(cut, seg_off, pd, pp, oracle.Params.make(3),
                                                    np.zeros(2, np.int32), np.zeros(2, np.uint8))
    assert gj.tolist() == [-1, -1] and jg.tolist() == [-1, -1] and rounds == 1 and stable == 1


def test_score_overflow_is_reported_not_wrapped(oracle):
    seg_off = np.array([0, 1], dtype=np.int64)
    dur = np.array([2**31 - 1], dtype=np.int32)
    mem = np.array([2**31 - 1], dtype=np.int32)
    safe = np.ones(1, dtype=np.uint8)
    progress = np.zeros(1, dtype=np.int32)
    W = np.array([2**31 - 1], dtype=np.int32)
    C = np.array([2**31 - 1], dtype=np.int32)
    pd, pp, cut = _tick(oracle, seg_off, dur, mem, safe, progress, W, C)
    with pytest.raises(RuntimeError):
        oracle.select(cut, seg_off, pd, pp, oracle.Params.make(1, wait_scale=2**31 - 1),
                      np.array([2**31 - 1], np.int32), np.zeros(1, np.uint8))


def test_mixed_breaks_fairness_ties_by_efficiency(oracle):
    """Two jobs of one class with equal fairness score 12 = 3*(2+2) = 4*(2+1):
    MIXED falls through to the larger F, FAIRNESS to the lower id."""
    seg_off = np.array([0, 1, 2], dtype=np.int64)
    dur = np.array([3, 4], dtype=np.int32)
    mem = np.array([1, 1], dtype=np.int32)
    safe = np.ones(2, dtype=np.uint8)
    progress = np.zeros(2, dtype=np.int32)
    W = np.array([10], dtype=np.int32)
    C = np.array([1], dtype=np.int32)
    wait = np.array([2, 1], dtype=np.int32)
    cls = np.array([1, 1], dtype=np.uint8)
    pd, pp, cut = _tick(oracle, seg_off, dur, mem, safe, progress, W, C)
    mixed = oracle.select(cut, seg_off, pd, pp, oracle.Params.make(3, wait_scale=2), wait, cls)
    fair = oracle.select(cut, seg_off, pd, pp, oracle.Params.make(1, wait_scale=2), wait, cls)
    assert (int(mixed[0][0]), int(mixed[2][0])) == (1, 12)
    assert (int(fair[0][0]), int(fair[2][0])) == (0, 12)


@pytest.mark.slow
def test_large_grant_digest_comes_from_this_oracle(oracle):
    """The stored digest of the Large config's grants under its round cap of 8
    (tests/golden/fullsize_digest_large.json, which the GPU test compares with) is what the
    oracle gives today: the whole Large tick recomputed here, about half a minute."""
    import importlib.util
    import json
    import os
    golden = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    with open(os.path.join(golden, "fullsize_digest_large.json")) as f:
        gold = json.load(f)
    spec = importlib.util.spec_from_file_location("make_fullsize_digest", os.path.join(golden, "make_fullsize_digest.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    wl = make_workload("large", gold["seed"])
    par = oracle.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override, 8)
    pd, pp, _ = oracle.prepare(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress)
    cut, _ = oracle.fit(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, wl.W, wl.C, False)
    res = oracle.resolve(cut, wl.seg_off, pd, pp, par, wl.wait, wl.sla_class)
    assert mod.grant_digest(*res) == gold["resolve"]["8"]
