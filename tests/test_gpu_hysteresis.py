"""GPU parity under the hysteresis rule on subdivision (sja_set_hysteresis; Sec. 3.9,
safeguard ii), against the CPU oracle: the cut matrix and interest bits, select, the
fused call, the rounds in both modes, the rule on top of admission limits and of the
area score, and a chain of ticks.  Integer work: bit-exact."""
import numpy as np
import pytest

from gen import make_channels, make_gaps, make_workload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def engine():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2509_19086_amd as P
    eng = P.Engine(0)
    yield eng
    eng.sja_set_hysteresis(None)
    eng.sja_set_limits(None)
    eng.sja_set_score(0)


def _cap_sets(wl):
    own = np.unique(wl.C).astype(np.int64)
    step = int(own[0])
    return {
        "gap_capacities": (own, step),                        # a gain of one slice size
        "gap_capacities_big_gain": (own, int(own[-1] - own[0])),
        "fine_set": (np.unique(np.concatenate([own // 4, own // 2, own, own * 2])), max(1, step // 4)),
        "set_below_the_peaks": (own[:2], 1),                  # long fragments have no cover at all
        "single": (own[-1:], 1),                              # nothing to gain: the plain fit
        "thirty_two": (np.unique(np.linspace(1, int(own[-1]), 32).astype(np.int64)), max(1, step // 8)),
    }


def hysteresis_tick_check(engine, oracle, wl, which, policies, fused, limits=False, area=False):
    import torch
    import paper_2509_19086_amd as P
    cap_set, min_gain = _cap_sets(wl)[which]
    assert len(cap_set) <= 32
    power, deadline = make_channels(wl, wl.seed)
    olim = d_power = d_deadline = None
    if limits:
        w_hi = int(wl.W.max())
        kw = dict(tau_min=max(1, w_hi // 14), tau_max=(2 * w_hi) // 3, power_cap=int(np.percentile(power, 85)), now=7)
        d_power, d_deadline = torch.from_numpy(power).cuda(), torch.from_numpy(deadline).cuda()
        engine.sja_set_limits(P.Limits.make(**kw), d_power, d_deadline)
        olim = oracle.Limits.make(**kw)
    engine.sja_set_score(1 if area else 0)
    engine.sja_set_hysteresis(cap_set, min_gain)
    try:
        t = P.DeviceTick(engine, wl, want_bits=not fused, want_cut=not fused)
        t.prepare()
        pd, pp, ps = oracle.prepare(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress)
        pa = oracle.area(wl.seg_off, wl.dur, wl.mem, wl.progress) if area else None
        cut, bits = oracle.fit_hysteresis(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, wl.W, wl.C, cap_set,
                                          min_gain, olim, power if limits else None,
                                          deadline if limits else None, True)
        plain, _ = oracle.fit_limited(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, wl.W, wl.C, olim,
                                      power if limits else None, deadline if limits else None)
        for policy in policies:
            par = P.Params.make(policy, wl.wait_scale, wl.sla_weight, wl.class0_override, wl.max_rounds)
            opar = oracle.Params.make(policy, wl.wait_scale, wl.sla_weight, wl.class0_override, wl.max_rounds)
            if fused:
                t.fit_select(par)
            else:
                t.fit(); t.select(par)
            torch.cuda.synchronize()
            # the caller-visible running tables do not depend on the rule
            np.testing.assert_array_equal(t.pre_dur.cpu().numpy().astype(np.int64), pd)
            np.testing.assert_array_equal(t.pre_peak.cpu().numpy().astype(np.int64), pp)
            np.testing.assert_array_equal(t.prev_safe.cpu().numpy(), ps)
            if not fused:
                np.testing.assert_array_equal(t.cut.cpu().numpy(), cut)
                np.testing.assert_array_equal(t.bits.cpu().numpy().view(np.uint32), bits)
            cj, cc, cs = oracle.select(cut, wl.seg_off, pd, pp, opar, wl.wait, wl.sla_class, pre_area=pa)
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
        return float((cut != plain).mean())
    finally:
        engine.sja_set_hysteresis(None)
        engine.sja_set_limits(None)
        engine.sja_set_score(0)


WHICH = ["gap_capacities", "gap_capacities_big_gain", "fine_set", "set_below_the_peaks", "single", "thirty_two"]


@pytest.mark.parametrize("which", WHICH)
def test_tiny_hysteresis(engine, oracle, which):
    for seed in (0, 2):
        hysteresis_tick_check(engine, oracle, make_workload("tiny", seed), which, [0, 1, 2, 3], False)
        hysteresis_tick_check(engine, oracle, make_workload("tiny", seed), which, [3], True)


@pytest.mark.parametrize("which", WHICH)
@pytest.mark.parametrize("fused", [False, True])
def test_small_hysteresis(engine, oracle, which, fused):
    moved = hysteresis_tick_check(engine, oracle, make_workload("small", 1), which, [0, 3], fused)
    if which == "single":
        assert moved == 0.0
    elif which != "gap_capacities_big_gain":
        assert moved > 0.01                                    # the rule did act


@pytest.mark.parametrize("fused", [False, True])
def test_medium_hysteresis(engine, oracle, fused):
    assert hysteresis_tick_check(engine, oracle, make_workload("medium", 0), "gap_capacities", [3], fused) > 0.01


@pytest.mark.parametrize("fused", [False, True])
def test_hysteresis_on_top_of_limits_and_area(engine, oracle, fused):
    wl = make_workload("small", 4)
    assert hysteresis_tick_check(engine, oracle, wl, "fine_set", [0, 2], fused, limits=True) > 0.005
    assert hysteresis_tick_check(engine, oracle, wl, "fine_set", [1, 3], fused, area=True) > 0.005
    assert hysteresis_tick_check(engine, oracle, wl, "gap_capacities", [3], fused, limits=True, area=True) > 0.005


@pytest.mark.parametrize("fused", [False, True])
def test_hysteresis_ragged(engine, oracle, fused):
    hysteresis_tick_check(engine, oracle, make_workload("stress", 7, n_gaps=333, n_jobs=1111), "fine_set", [3, 0], fused)
    hysteresis_tick_check(engine, oracle, make_workload("large", 7, n_gaps=130, n_jobs=70), "gap_capacities", [0], fused)
    hysteresis_tick_check(engine, oracle, make_workload("medium", 5, n_gaps=1, n_jobs=1), "fine_set", [2], fused)


def test_rule_takes_effect_at_prepare_and_clears_again(engine, oracle):
    import torch
    import paper_2509_19086_amd as P
    wl = make_workload("small", 3)
    cap_set, min_gain = _cap_sets(wl)["gap_capacities"]
    t = P.DeviceTick(engine, wl, want_bits=False)
    plain, _ = oracle.fit(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, wl.W, wl.C, False)
    want, _ = oracle.fit_hysteresis(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, wl.W, wl.C, cap_set, min_gain)
    assert (want != plain).mean() > 0.01
    try:
        t.prepare()
        engine.sja_set_hysteresis(cap_set, min_gain)
        t.fit(); torch.cuda.synchronize()                      # set after the prepare: not yet in force
        np.testing.assert_array_equal(t.cut.cpu().numpy(), plain)
        t.prepare(); t.fit(); torch.cuda.synchronize()
        np.testing.assert_array_equal(t.cut.cpu().numpy(), want)
        engine.sja_set_hysteresis(None)
        t.fit(); torch.cuda.synchronize()                      # cleared: still in force until the next prepare
        np.testing.assert_array_equal(t.cut.cpu().numpy(), want)
        t.prepare(); t.fit(); torch.cuda.synchronize()
        np.testing.assert_array_equal(t.cut.cpu().numpy(), plain)
        for bad in (([2, 1], 1), ([1, 2], 0), (list(range(33)), 1)):
            with pytest.raises(RuntimeError):
                engine.sja_set_hysteresis(*bad)
    finally:
        engine.sja_set_hysteresis(None)


def test_chain_of_ticks_under_hysteresis(engine, oracle):
    """sja_advance rebuilds the moved jobs under the rule their prepare used, and leaves the
    others' tables as they are."""
    import torch
    import paper_2509_19086_amd as P
    wl = make_workload("small", 6)
    cap_set, min_gain = _cap_sets(wl)["gap_capacities"]
    par = P.Params.make(3, wl.wait_scale, wl.sla_weight, wl.class0_override, 0)
    opar = oracle.Params.make(3, wl.wait_scale, wl.sla_weight, wl.class0_override, 0)
    t = P.DeviceTick(engine, wl, want_bits=False, want_cut=True)
    engine.sja_set_hysteresis(cap_set, min_gain)
    try:
        t.prepare()
        engine.sja_set_hysteresis(None)                        # the chain keeps the rule of its prepare
        progress, wait = wl.progress.copy(), wl.wait.copy()
        moved = shortened = 0
        for tick in range(5):
            W, C = (wl.W, wl.C) if tick == 0 else make_gaps("small", 6, tick)
            t.set_gaps(W, C)
            if tick % 2:
                t.fit(); t.select(par)
            else:
                t.fit_select(par)
            t.resolve(par)
            pd, pp, _ = oracle.prepare(wl.seg_off, wl.dur, wl.mem, wl.safe, progress)
            cut, _ = oracle.fit_hysteresis(wl.seg_off, wl.dur, wl.mem, wl.safe, progress, W, C, cap_set, min_gain)
            plain, _ = oracle.fit(wl.seg_off, wl.dur, wl.mem, wl.safe, progress, W, C, False)
            shortened += int((cut != plain).sum())
            if tick % 2:
                np.testing.assert_array_equal(t.cut.cpu().numpy(), cut, err_msg=f"tick {tick}")
            gj, gc, gs, jg, rounds, stable = oracle.resolve(cut, wl.seg_off, pd, pp, opar, wait, wl.sla_class)
            np.testing.assert_array_equal(t.grant_job.cpu().numpy(), gj, err_msg=f"tick {tick}")
            np.testing.assert_array_equal(t.grant_cut.cpu().numpy(), gc, err_msg=f"tick {tick}")
            np.testing.assert_array_equal(t.grant_score.cpu().numpy(), gs, err_msg=f"tick {tick}")
            t.advance(1000)
            torch.cuda.synchronize()
            p2, w2, m = oracle.advance(wl.seg_off, pd, pp, W, C, gj, gc, jg, progress, wait, 1000)
            np.testing.assert_array_equal(t.progress.cpu().numpy(), p2)
            assert t.metrics.cpu().tolist() == m.tolist()
            moved += int(m[2])
            progress, wait = p2, w2
        assert moved > 100 and shortened > 1000
    finally:
        engine.sja_set_hysteresis(None)
