"""GPU parity with the area-under-the-envelope score (sja_set_score), against the CPU oracle:
select, the fused call, the rounds in both modes and a chain of ticks.  Integer work: bit-exact."""
import numpy as np
import pytest

from gen import make_gaps, make_workload

pytestmark = pytest.mark.gpu

AREA, RECTANGLE = 1, 0


@pytest.fixture(scope="module")
def engine():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2509_19086_amd as P
    eng = P.Engine(0)
    yield eng
    eng.sja_set_score(RECTANGLE)


def area_tick_check(engine, oracle, wl, policies, fused):
    import torch
    import paper_2509_19086_amd as P
    engine.sja_set_score(AREA)
    try:
        t = P.DeviceTick(engine, wl, want_bits=False, want_cut=not fused)
        t.prepare()
        pd, pp, _ = oracle.prepare(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress)
        pa = oracle.area(wl.seg_off, wl.dur, wl.mem, wl.progress)
        cut, _ = oracle.fit(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, wl.W, wl.C, False)
        differs = False
        for policy in policies:
            par = P.Params.make(policy, wl.wait_scale, wl.sla_weight, wl.class0_override, wl.max_rounds)
            opar = oracle.Params.make(policy, wl.wait_scale, wl.sla_weight, wl.class0_override, wl.max_rounds)
            if fused:
                t.fit_select(par)
            else:
                t.fit(); t.select(par)
            torch.cuda.synchronize()
            cj, cc, cs = oracle.select(cut, wl.seg_off, pd, pp, opar, wl.wait, wl.sla_class, pre_area=pa)
            rj, _, rs = oracle.select(cut, wl.seg_off, pd, pp, opar, wl.wait, wl.sla_class)
            differs = differs or bool((cj != rj).any() or (cs != rs).any())
            np.testing.assert_array_equal(t.cand_job.cpu().numpy(), cj, err_msg=f"policy {policy}")
            np.testing.assert_array_equal(t.cand_cut.cpu().numpy(), cc, err_msg=f"policy {policy}")
            np.testing.assert_array_equal(t.cand_score.cpu().numpy(), cs, err_msg=f"policy {policy}")
            want = oracle.resolve(cut, wl.seg_off, pd, pp, opar, wl.wait, wl.sla_class, pre_area=pa)
            for mode in ((0,) if fused else (0, 1)):
                try:
                    engine.sja_set_resolve_mode(mode)
                    for out in (t.grant_job, t.grant_cut, t.grant_score, t.job_gap):
                        out.fill_(-5)
                    t.resolve(par)
                finally:
                    engine.sja_set_resolve_mode(0)
                got = (t.grant_job, t.grant_cut, t.grant_score, t.job_gap)
                for x, y in zip(got, want[:4]):
                    np.testing.assert_array_equal(x.cpu().numpy(), y, err_msg=f"policy {policy} mode {mode}")
                assert t.rounds.cpu().tolist() == [want[4], want[5]]
        return differs
    finally:
        engine.sja_set_score(RECTANGLE)


@pytest.mark.parametrize("fused", [False, True])
@pytest.mark.parametrize("name,seed", [("tiny", 0), ("tiny", 2), ("small", 1), ("medium", 0)])
def test_area_score(engine, oracle, name, seed, fused):
    differs = area_tick_check(engine, oracle, make_workload(name, seed), [0, 1, 2, 3], fused)
    assert differs                                             # the two readings rank differently on these inputs


@pytest.mark.parametrize("fused", [False, True])
def test_area_score_ragged(engine, oracle, fused):
    area_tick_check(engine, oracle, make_workload("stress", 7, n_gaps=333, n_jobs=1111), [3, 0], fused)
    area_tick_check(engine, oracle, make_workload("large", 7, n_gaps=130, n_jobs=70), [0], fused)
    area_tick_check(engine, oracle, make_workload("medium", 5, n_gaps=1, n_jobs=1), [2], fused)


def test_area_score_chain_of_ticks_and_back(engine, oracle):
    import torch
    import paper_2509_19086_amd as P
    wl = make_workload("small", 8)
    par = P.Params.make(3, wl.wait_scale, wl.sla_weight, wl.class0_override, 0)
    opar = oracle.Params.make(3, wl.wait_scale, wl.sla_weight, wl.class0_override, 0)
    t = P.DeviceTick(engine, wl, want_bits=False, want_cut=False)
    engine.sja_set_score(AREA)
    try:
        t.prepare()
        engine.sja_set_score(RECTANGLE)                        # the chain keeps the score of its prepare
        progress, wait = wl.progress.copy(), wl.wait.copy()
        for tick in range(4):
            W, C = (wl.W, wl.C) if tick == 0 else make_gaps("small", 8, tick)
            t.set_gaps(W, C)
            t.fit_select(par); t.resolve(par)
            pd, pp, _ = oracle.prepare(wl.seg_off, wl.dur, wl.mem, wl.safe, progress)
            pa = oracle.area(wl.seg_off, wl.dur, wl.mem, progress)
            cut, _ = oracle.fit(wl.seg_off, wl.dur, wl.mem, wl.safe, progress, W, C, False)
            gj, gc, gs, jg, rounds, stable = oracle.resolve(cut, wl.seg_off, pd, pp, opar, wait, wl.sla_class,
                                                            pre_area=pa)
            np.testing.assert_array_equal(t.grant_job.cpu().numpy(), gj, err_msg=f"tick {tick}")
            np.testing.assert_array_equal(t.grant_score.cpu().numpy(), gs, err_msg=f"tick {tick}")
            t.advance(1000)
            torch.cuda.synchronize()
            p2, w2, m = oracle.advance(wl.seg_off, pd, pp, W, C, gj, gc, jg, progress, wait, 1000)
            np.testing.assert_array_equal(t.progress.cpu().numpy(), p2)
            assert t.metrics.cpu().tolist() == m.tolist()      # the tick's totals stay the rectangle's
            progress, wait = p2, w2
        # a new prepare goes back to the default score
        t2 = P.DeviceTick(engine, wl, want_bits=False, want_cut=False)
        t2.prepare(); t2.fit_select(par)
        torch.cuda.synchronize()
        pd, pp, _ = oracle.prepare(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress)
        cut, _ = oracle.fit(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, wl.W, wl.C, False)
        cj, cc, cs = oracle.select(cut, wl.seg_off, pd, pp, opar, wl.wait, wl.sla_class)
        np.testing.assert_array_equal(t2.cand_job.cpu().numpy(), cj)
        np.testing.assert_array_equal(t2.cand_score.cpu().numpy(), cs)
    finally:
        engine.sja_set_score(RECTANGLE)
    with pytest.raises(RuntimeError):
        engine.sja_set_score(2)


def test_area_score_under_admission_limits(engine, oracle):
    """Both options at once: atoms filtered by the limits carry their areas along."""
    import torch
    import paper_2509_19086_amd as P
    from gen import make_channels
    wl = make_workload("small", 5)
    power, deadline = make_channels(wl, 5)
    kw = dict(tau_min=120, tau_max=1300, power_cap=int(np.percentile(power, 85)), now=4)
    par = P.Params.make(3, wl.wait_scale, wl.sla_weight, wl.class0_override, 0)
    opar = oracle.Params.make(3, wl.wait_scale, wl.sla_weight, wl.class0_override, 0)
    d_power, d_deadline = torch.from_numpy(power).cuda(), torch.from_numpy(deadline).cuda()
    engine.sja_set_score(AREA)
    engine.sja_set_limits(P.Limits.make(**kw), d_power, d_deadline)
    try:
        pd, pp, _ = oracle.prepare(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress)
        pa = oracle.area(wl.seg_off, wl.dur, wl.mem, wl.progress)
        cut, _ = oracle.fit_limited(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, wl.W, wl.C,
                                    oracle.Limits.make(**kw), power, deadline)
        want = oracle.resolve(cut, wl.seg_off, pd, pp, opar, wl.wait, wl.sla_class, pre_area=pa)
        cj, cc, cs = oracle.select(cut, wl.seg_off, pd, pp, opar, wl.wait, wl.sla_class, pre_area=pa)
        for fused in (False, True):
            t = P.DeviceTick(engine, wl, want_bits=False, want_cut=not fused)
            t.prepare()
            if fused:
                t.fit_select(par)
            else:
                t.fit(); t.select(par)
                np.testing.assert_array_equal(t.cut.cpu().numpy(), cut)
            np.testing.assert_array_equal(t.cand_job.cpu().numpy(), cj)
            np.testing.assert_array_equal(t.cand_score.cpu().numpy(), cs)
            t.resolve(par)
            for x, y in zip((t.grant_job, t.grant_cut, t.grant_score, t.job_gap), want[:4]):
                np.testing.assert_array_equal(x.cpu().numpy(), y)
            assert t.rounds.cpu().tolist() == [want[4], want[5]]
    finally:
        engine.sja_set_limits(None)
        engine.sja_set_score(RECTANGLE)
