"""GPU checks at the full sizes of the two largest configs, in the launch
configuration bench.py times, that go beyond the element-by-element comparison
of fit and select in tests/test_gpu_fullsize_elementwise.py: the grants (their
invariants, which hold at any size, with the oracle evaluating every granted
pair; digests of the oracle's own grants), both implementations of the rounds
against each other, chains of ticks, admission limits, the area score, and a
batch whose element offsets pass 2^32."""
import numpy as np
import pytest

from gen import make_workload

pytestmark = [pytest.mark.gpu, pytest.mark.slow]


def _check_full_size(oracle, name, n_pairs, n_rows, max_rounds, until_stable=False):
    import torch
    import paper_2509_19086_amd as P
    wl = make_workload(name, 0)
    wl.max_rounds = max_rounds
    G, J = wl.n_gaps, wl.n_jobs
    eng = P.Engine(0)
    t = P.DeviceTick(eng, wl)
    par = P.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override, max_rounds)
    opar = oracle.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override, max_rounds)
    t.prepare(); t.fit(); t.select(par)
    torch.cuda.synchronize()

    # prepare: whole arrays (cheap on the CPU)
    pd, pp, ps = oracle.prepare(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress)
    np.testing.assert_array_equal(t.pre_dur.cpu().numpy().astype(np.int64), pd)
    np.testing.assert_array_equal(t.pre_peak.cpu().numpy().astype(np.int64), pp)
    np.testing.assert_array_equal(t.prev_safe.cpu().numpy(), ps)

    # fit: sampled pairs anywhere in the matrix
    rng = np.random.default_rng(42)
    gi = rng.integers(0, G, size=n_pairs).astype(np.int32)
    ji = rng.integers(0, J, size=n_pairs).astype(np.int32)
    gi[:4] = [0, G - 1, 0, G - 1]
    ji[:4] = [0, J - 1, J - 1, 0]
    want, _, _ = oracle.fit_pairs(gi, ji, wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, wl.W, wl.C)
    flat = torch.from_numpy(gi.astype(np.int64) * J + ji.astype(np.int64)).cuda()
    got = t.cut.view(-1)[flat].cpu().numpy()
    np.testing.assert_array_equal(got, want)

    # fit, interest rows and select: whole rows of sampled gaps (first, last, extremes, random)
    rows = np.unique(np.concatenate([[0, G - 1, int(np.argmin(wl.W)), int(np.argmax(wl.W))],
                                     rng.integers(0, G, size=n_rows)])).astype(np.int64)
    Wr = np.ascontiguousarray(wl.W[rows]); Cr = np.ascontiguousarray(wl.C[rows])
    cut_r, bits_r = oracle.fit(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, Wr, Cr)
    rows_t = torch.from_numpy(rows).cuda()
    np.testing.assert_array_equal(t.cut[rows_t].cpu().numpy(), cut_r)
    np.testing.assert_array_equal(t.bits[rows_t].cpu().numpy().view(np.uint32), bits_r)
    cj, cc, cs = oracle.select(cut_r, wl.seg_off, pd, pp, opar, wl.wait, wl.sla_class)
    np.testing.assert_array_equal(t.cand_job[rows_t].cpu().numpy(), cj)
    np.testing.assert_array_equal(t.cand_cut[rows_t].cpu().numpy(), cc)
    np.testing.assert_array_equal(t.cand_score[rows_t].cpu().numpy(), cs)

    # resolve: invariants that hold at any size, with the oracle evaluating each granted pair
    def check_grants(cap):
        p = P.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override, cap)
        t.resolve(p)
        gj = t.grant_job.cpu().numpy(); gc = t.grant_cut.cpu().numpy(); gs = t.grant_score.cpu().numpy()
        jg = t.job_gap.cpu().numpy()
        rounds, stable = t.rounds.cpu().tolist()
        granted = np.nonzero(gj >= 0)[0]
        assert len(granted) > 0
        assert len(np.unique(gj[granted])) == len(granted)                  # no job holds two gaps
        np.testing.assert_array_equal(jg[gj[granted]], granted)             # job_gap inverts grant_job
        assert (jg >= 0).sum() == len(granted)
        ocut, sd, sp = oracle.fit_pairs(granted.astype(np.int32), gj[granted], wl.seg_off, wl.dur,
                                        wl.mem, wl.safe, wl.progress, wl.W, wl.C)
        np.testing.assert_array_equal(gc[granted], ocut)                    # an interested pair, same cut
        assert (ocut >= 0).all()
        assert (sd <= wl.W[granted]).all() and (sp <= wl.C[granted]).all()  # fits by construction
        F = sd * sp
        wait = wl.wait[gj[granted]].astype(np.int64)
        cls = wl.sla_class[gj[granted]]
        score = {0: F, 1: F * (wl.wait_scale + wait), 2: F * np.asarray(wl.sla_weight, np.int64)[cls],
                 3: F * (wl.wait_scale + wait)}[wl.policy]
        np.testing.assert_array_equal(gs[granted], score)
        assert (gs[gj < 0] == 0).all() and (gc[gj < 0] == -1).all()
        if 0 in rows:                                                        # gap 0 always keeps its first choice
            assert gj[0] == cj[0] and gc[0] == cc[0] and gs[0] == cs[0]
        assert 1 <= rounds <= (cap if cap else min(G, J) + 1)
        if not (cap and rounds == cap and stable == 0):
            assert stable == 1
            # stable: a sampled ungranted gap has no un-held interested job left
            ung = [i for i, g in enumerate(rows) if gj[g] < 0]
            if ung:
                sub = cut_r[ung]
                rj, _, _ = oracle.select(sub, wl.seg_off, pd, pp, opar, wl.wait, wl.sla_class, jg)
                assert (rj == -1).all()
        return gj, gc, gs, jg, rounds, stable

    # the fused call reports the same candidates as sja_select after sja_fit, for every gap
    sel = (t.cand_job.clone(), t.cand_cut.clone(), t.cand_score.clone())
    for out in (t.cand_job, t.cand_cut, t.cand_score):
        out.fill_(-5)
    t.fit_select(par)
    torch.cuda.synchronize()
    for a, b in zip(sel, (t.cand_job, t.cand_cut, t.cand_score)):
        assert torch.equal(a, b)
    np.testing.assert_array_equal(t.cand_job[rows_t].cpu().numpy(), cj)
    t.fit()                                   # the cut matrix again, for the matrix-scanning rounds below
    torch.cuda.synchronize()

    first = check_grants(max_rounds)
    # the two implementations of the rounds agree bit for bit at full size
    try:
        eng.sja_set_resolve_mode(1)
        other = check_grants(max_rounds)
    finally:
        eng.sja_set_resolve_mode(0)
    for a, b in zip(first, other):
        np.testing.assert_array_equal(a, b)
    if until_stable:
        t.fit_select(par)                     # resolve on top of the fused call: no cut matrix involved
        gj, _, _, _, rounds, stable = check_grants(0)
        assert stable == 1 and rounds > max_rounds
        # with the cap gone nothing granted before is taken back
        keep = first[0] >= 0
        np.testing.assert_array_equal(gj[keep], first[0][keep])


def test_large_full_size(oracle):
    _check_full_size(oracle, "large", n_pairs=400_000, n_rows=24, max_rounds=8)


def test_stress_full_size(oracle):
    _check_full_size(oracle, "stress", n_pairs=300_000, n_rows=12, max_rounds=8, until_stable=True)


def test_stress_chain_of_ticks(oracle):
    """Three ticks at the full Stress size: fused fit-select, grants until stable, advance.
    Each tick the oracle evaluates every granted pair from the progress points it tracks itself,
    which fixes the cuts, the filled area and the new progress points; whole running tables are
    compared after each advance, and sampled gap rows pin the next tick's candidates."""
    import torch
    import paper_2509_19086_amd as P
    from gen import make_gaps
    wl = make_workload("stress", 0)
    G, J = wl.n_gaps, wl.n_jobs
    lens = np.diff(wl.seg_off)
    eng = P.Engine(0)
    t = P.DeviceTick(eng, wl, want_bits=False, want_cut=False)
    par = P.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override, 0)
    opar = oracle.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override, 0)
    t.prepare()
    progress, wait = wl.progress.copy(), wl.wait.copy()
    rng = np.random.default_rng(5)
    job_of_seg = np.repeat(np.arange(J), lens)
    k_in_job = np.arange(int(wl.seg_off[-1])) - wl.seg_off[:-1][job_of_seg]
    for tick in range(3):
        W, C = (wl.W, wl.C) if tick == 0 else make_gaps("stress", 0, tick)
        t.set_gaps(W, C)
        t.fit_select(par)
        torch.cuda.synchronize()
        pd, pp, ps = oracle.prepare(wl.seg_off, wl.dur, wl.mem, wl.safe, progress)
        rows = np.unique(np.concatenate([[0, G - 1], rng.integers(0, G, size=6)])).astype(np.int64)
        cut_r, _ = oracle.fit(wl.seg_off, wl.dur, wl.mem, wl.safe, progress,
                              np.ascontiguousarray(W[rows]), np.ascontiguousarray(C[rows]), False)
        cj, cc, cs = oracle.select(cut_r, wl.seg_off, pd, pp, opar, wait, wl.sla_class)
        rows_t = torch.from_numpy(rows).cuda()
        np.testing.assert_array_equal(t.cand_job[rows_t].cpu().numpy(), cj, err_msg=f"tick {tick}")
        np.testing.assert_array_equal(t.cand_cut[rows_t].cpu().numpy(), cc, err_msg=f"tick {tick}")
        np.testing.assert_array_equal(t.cand_score[rows_t].cpu().numpy(), cs, err_msg=f"tick {tick}")

        t.resolve(par)
        gj = t.grant_job.cpu().numpy(); gc = t.grant_cut.cpu().numpy(); jg = t.job_gap.cpu().numpy()
        assert t.rounds.cpu().tolist()[1] == 1
        granted = np.nonzero(gj >= 0)[0]
        assert len(granted) > 0 and len(np.unique(gj[granted])) == len(granted)
        np.testing.assert_array_equal(jg[gj[granted]], granted)
        assert (jg >= 0).sum() == len(granted)
        ocut, sd, sp = oracle.fit_pairs(granted.astype(np.int32), gj[granted], wl.seg_off, wl.dur, wl.mem,
                                        wl.safe, progress, W, C)
        np.testing.assert_array_equal(gc[granted], ocut)
        assert gj[0] == cj[0] and gc[0] == cc[0]               # gap 0 keeps its first choice

        t.advance(1000)
        torch.cuda.synchronize()
        p2, w2, m = oracle.advance(wl.seg_off, pd, pp, W, C, gj, gc, jg, progress, wait, 1000)
        assert m[0] == int((sd * sp).sum())                     # the oracle's own two routes agree
        np.testing.assert_array_equal(t.progress.cpu().numpy(), p2)
        np.testing.assert_array_equal(t.wait.cpu().numpy(), w2)
        assert t.metrics.cpu().tolist() == m.tolist()
        progress, wait = p2, w2
        pd2, pp2, ps2 = oracle.prepare(wl.seg_off, wl.dur, wl.mem, wl.safe, progress)
        live = k_in_job >= progress[job_of_seg]
        np.testing.assert_array_equal(t.pre_dur.cpu().numpy().astype(np.int64)[live], pd2[live])
        np.testing.assert_array_equal(t.pre_peak.cpu().numpy().astype(np.int64)[live], pp2[live])
        np.testing.assert_array_equal(t.prev_safe.cpu().numpy()[live], ps2[live])


def test_stress_limits_full_size(oracle):
    """The full Stress tick under all admission limits at once: sampled pairs and whole sampled
    rows of the cut matrix, the fused candidates for every gap, and the grants with the oracle
    evaluating each granted pair under the same limits."""
    import torch
    import paper_2509_19086_amd as P
    from gen import make_channels
    wl = make_workload("stress", 0)
    G, J = wl.n_gaps, wl.n_jobs
    power, deadline = make_channels(wl, 0)
    kw = dict(tau_min=int(wl.W.max()) // 14, tau_max=(2 * int(wl.W.max())) // 3,
              power_cap=int(np.percentile(power, 85)), now=7)
    eng = P.Engine(0)
    t = P.DeviceTick(eng, wl, want_bits=True)
    d_power, d_deadline = torch.from_numpy(power).cuda(), torch.from_numpy(deadline).cuda()
    eng.sja_set_limits(P.Limits.make(**kw), d_power, d_deadline)
    olim = oracle.Limits.make(**kw)
    par = P.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override, 0)
    opar = oracle.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override, 0)
    t.prepare(); t.fit(); t.select(par)
    torch.cuda.synchronize()

    rng = np.random.default_rng(43)
    gi = rng.integers(0, G, size=300_000).astype(np.int32)
    ji = rng.integers(0, J, size=300_000).astype(np.int32)
    want, _, _ = oracle.fit_pairs_limited(gi, ji, wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, wl.W, wl.C,
                                          olim, power, deadline)
    plain, _, _ = oracle.fit_pairs(gi, ji, wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, wl.W, wl.C)
    assert (want != plain).mean() > 0.05                       # the limits bind
    flat = torch.from_numpy(gi.astype(np.int64) * J + ji.astype(np.int64)).cuda()
    np.testing.assert_array_equal(t.cut.view(-1)[flat].cpu().numpy(), want)

    rows = np.unique(np.concatenate([[0, G - 1, int(np.argmax(wl.W))], rng.integers(0, G, size=8)])).astype(np.int64)
    cut_r, bits_r = oracle.fit_limited(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress,
                                       np.ascontiguousarray(wl.W[rows]), np.ascontiguousarray(wl.C[rows]),
                                       olim, power, deadline, True)
    rows_t = torch.from_numpy(rows).cuda()
    np.testing.assert_array_equal(t.cut[rows_t].cpu().numpy(), cut_r)
    np.testing.assert_array_equal(t.bits[rows_t].cpu().numpy().view(np.uint32), bits_r)
    pd, pp, _ = oracle.prepare(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress)
    cj, cc, cs = oracle.select(cut_r, wl.seg_off, pd, pp, opar, wl.wait, wl.sla_class)
    np.testing.assert_array_equal(t.cand_job[rows_t].cpu().numpy(), cj)
    np.testing.assert_array_equal(t.cand_score[rows_t].cpu().numpy(), cs)

    sel = (t.cand_job.clone(), t.cand_cut.clone(), t.cand_score.clone())
    t.fit_select(par)
    torch.cuda.synchronize()
    for a, b in zip(sel, (t.cand_job, t.cand_cut, t.cand_score)):
        assert torch.equal(a, b)

    t.resolve(par)
    gj = t.grant_job.cpu().numpy(); gc = t.grant_cut.cpu().numpy(); jg = t.job_gap.cpu().numpy()
    granted = np.nonzero(gj >= 0)[0]
    assert len(granted) > 1000 and len(np.unique(gj[granted])) == len(granted)
    np.testing.assert_array_equal(jg[gj[granted]], granted)
    ocut, sd, sp = oracle.fit_pairs_limited(granted.astype(np.int32), gj[granted], wl.seg_off, wl.dur, wl.mem,
                                            wl.safe, wl.progress, wl.W, wl.C, olim, power, deadline)
    np.testing.assert_array_equal(gc[granted], ocut)
    lens = np.diff(wl.seg_off)
    assert (sd <= kw["tau_max"]).all() and (sd <= deadline[gj[granted]].astype(np.int64) - kw["now"]).all()
    assert ((sd >= kw["tau_min"]) | (ocut == lens[gj[granted]])).all()
    assert gj[0] == cj[0] and gc[0] == cc[0]


@pytest.mark.parametrize("name", ["large", "stress"])
def test_grants_match_the_oracle_digests(name):
    """The grants of every gap at full size, with the round cap 8 and until stable, against
    digests of the oracle's grants written ahead of time (tests/golden/make_fullsize_digest.py:
    2007 rounds at Large, 9567 at Stress, hours of oracle time).  Fit and select are compared
    element by element in tests/test_gpu_fullsize_elementwise.py; only the grants, which the
    oracle cannot recompute inside a test, go through digests."""
    import json
    import os
    import torch
    import paper_2509_19086_amd as P
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", f"fullsize_digest_{name}.json")
    with open(path) as f:
        gold = json.load(f)
    wl = make_workload(name, gold["seed"])
    assert (wl.n_gaps, wl.n_jobs, int(wl.policy)) == (gold["n_gaps"], gold["n_jobs"], gold["policy"])
    eng = P.Engine(0)
    t = P.DeviceTick(eng, wl, want_bits=False)
    par = P.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override, 0)
    t.prepare(); t.fit(); t.select(par)
    torch.cuda.synchronize()
    gw = torch.arange(1, wl.n_gaps + 1, dtype=torch.int64, device="cuda:0")
    jw = torch.arange(1, wl.n_jobs + 1, dtype=torch.int64, device="cuda:0")
    assert gold.get("resolve")
    # mode 0: the lists as they are built by default; mode 2: the form in which the records' jobs
    # are looked up through their ranks (what very large batches get by themselves)
    try:
        for mode in (0, 2):
            eng.sja_set_resolve_mode(mode)
            for cap, want in gold["resolve"].items():
                for out in (t.grant_job, t.grant_cut, t.grant_score, t.job_gap, t.rounds):
                    out.fill_(-5)
                t.resolve(P.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override, int(cap)))
                rounds, stable = t.rounds.cpu().tolist()
                got_r = {"rounds": rounds, "stable": stable, "grants": int((t.grant_job >= 0).sum().item()),
                         "grant_job": int((t.grant_job.to(torch.int64) * gw).sum().item()),
                         "grant_cut": int((t.grant_cut.to(torch.int64) * gw).sum().item()),
                         "grant_score": int(t.grant_score.sum().item()),
                         "job_gap": int((t.job_gap.to(torch.int64) * jw).sum().item())}
                assert got_r == want, f"round cap {cap}, mode {mode}"
    finally:
        eng.sja_set_resolve_mode(0)


def test_beyond_stress_64bit_indexing(oracle):
    """49152 gaps x 131072 jobs = 6.4e9 pairs (a 25.8 GB cut matrix): element offsets pass 2^32.
    Sampled pairs (the last element among them), whole sampled rows (the last row among them),
    the fused candidates for every gap, and the grants of a capped resolve in both modes."""
    import torch
    import paper_2509_19086_amd as P
    wl = make_workload("stress", 3, n_gaps=49152, n_jobs=131072)
    G, J = wl.n_gaps, wl.n_jobs
    assert G * J > 2**32
    eng = P.Engine(0)
    t = P.DeviceTick(eng, wl, want_bits=True)
    par = P.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override, 8)
    opar = oracle.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override, 8)
    t.prepare(); t.fit(); t.select(par)
    torch.cuda.synchronize()
    rng = np.random.default_rng(44)
    gi = rng.integers(0, G, size=300_000).astype(np.int32)
    ji = rng.integers(0, J, size=300_000).astype(np.int32)
    gi[:6] = [0, G - 1, 0, G - 1, G // 2, 32768]
    ji[:6] = [0, J - 1, J - 1, 0, J // 2, 65536]
    want, _, _ = oracle.fit_pairs(gi, ji, wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, wl.W, wl.C)
    flat = torch.from_numpy(gi.astype(np.int64) * J + ji.astype(np.int64)).cuda()
    np.testing.assert_array_equal(t.cut.view(-1)[flat].cpu().numpy(), want)

    rows = np.unique(np.concatenate([[0, G - 1, 32767, 32768], rng.integers(0, G, size=6)])).astype(np.int64)
    cut_r, bits_r = oracle.fit(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress,
                               np.ascontiguousarray(wl.W[rows]), np.ascontiguousarray(wl.C[rows]))
    rows_t = torch.from_numpy(rows).cuda()
    np.testing.assert_array_equal(t.cut[rows_t].cpu().numpy(), cut_r)
    np.testing.assert_array_equal(t.bits[rows_t].cpu().numpy().view(np.uint32), bits_r)
    pd, pp, _ = oracle.prepare(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress)
    cj, cc, cs = oracle.select(cut_r, wl.seg_off, pd, pp, opar, wl.wait, wl.sla_class)
    np.testing.assert_array_equal(t.cand_job[rows_t].cpu().numpy(), cj)
    np.testing.assert_array_equal(t.cand_cut[rows_t].cpu().numpy(), cc)
    np.testing.assert_array_equal(t.cand_score[rows_t].cpu().numpy(), cs)

    sel = (t.cand_job.clone(), t.cand_cut.clone(), t.cand_score.clone())
    outs = []
    try:
        for mode in (0, 1):
            eng.sja_set_resolve_mode(mode)
            t.resolve(par)
            outs.append([x.cpu().numpy().copy() for x in (t.grant_job, t.grant_cut, t.grant_score, t.job_gap, t.rounds)])
    finally:
        eng.sja_set_resolve_mode(0)
    for a, b in zip(*outs):
        np.testing.assert_array_equal(a, b)
    gj, gc = outs[0][0], outs[0][1]
    granted = np.nonzero(gj >= 0)[0]
    assert len(granted) > 1000 and len(np.unique(gj[granted])) == len(granted)
    ocut, _, _ = oracle.fit_pairs(granted.astype(np.int32), gj[granted], wl.seg_off, wl.dur, wl.mem, wl.safe,
                                  wl.progress, wl.W, wl.C)
    np.testing.assert_array_equal(gc[granted], ocut)
    t.fit_select(par)
    torch.cuda.synchronize()
    for a, b in zip(sel, (t.cand_job, t.cand_cut, t.cand_score)):
        assert torch.equal(a, b)


def test_stress_area_score_full_size(oracle):
    """The area score at the full Stress size: candidates of sampled gap rows against the oracle,
    the fused call against select for every gap, and every grant's score recomputed by the oracle."""
    import torch
    import paper_2509_19086_amd as P
    wl = make_workload("stress", 0)
    G, J = wl.n_gaps, wl.n_jobs
    eng = P.Engine(0)
    eng.sja_set_score(1)
    t = P.DeviceTick(eng, wl, want_bits=False)
    par = P.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override, 8)
    opar = oracle.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override, 8)
    t.prepare(); t.fit(); t.select(par)
    torch.cuda.synchronize()
    pd, pp, _ = oracle.prepare(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress)
    pa = oracle.area(wl.seg_off, wl.dur, wl.mem, wl.progress)
    rng = np.random.default_rng(45)
    rows = np.unique(np.concatenate([[0, G - 1], rng.integers(0, G, size=10)])).astype(np.int64)
    cut_r, _ = oracle.fit(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress,
                          np.ascontiguousarray(wl.W[rows]), np.ascontiguousarray(wl.C[rows]), False)
    cj, cc, cs = oracle.select(cut_r, wl.seg_off, pd, pp, opar, wl.wait, wl.sla_class, pre_area=pa)
    rj, _, rs = oracle.select(cut_r, wl.seg_off, pd, pp, opar, wl.wait, wl.sla_class)
    assert (cs != rs).any()                                    # not the rectangle's scores
    rows_t = torch.from_numpy(rows).cuda()
    np.testing.assert_array_equal(t.cand_job[rows_t].cpu().numpy(), cj)
    np.testing.assert_array_equal(t.cand_cut[rows_t].cpu().numpy(), cc)
    np.testing.assert_array_equal(t.cand_score[rows_t].cpu().numpy(), cs)
    sel = (t.cand_job.clone(), t.cand_cut.clone(), t.cand_score.clone())
    t.resolve(par)
    gj = t.grant_job.cpu().numpy(); gc = t.grant_cut.cpu().numpy(); gs = t.grant_score.cpu().numpy()
    granted = np.nonzero(gj >= 0)[0]
    assert len(granted) > 1000 and len(np.unique(gj[granted])) == len(granted)
    ocut, _, _ = oracle.fit_pairs(granted.astype(np.int32), gj[granted], wl.seg_off, wl.dur, wl.mem, wl.safe,
                                  wl.progress, wl.W, wl.C)
    np.testing.assert_array_equal(gc[granted], ocut)
    F = pa[wl.seg_off[:-1][gj[granted]] + ocut - 1]
    np.testing.assert_array_equal(gs[granted], F * (wl.wait_scale + wl.wait[gj[granted]].astype(np.int64)))
    assert gj[0] == cj[0] and gs[0] == cs[0]
    t.fit_select(par)
    torch.cuda.synchronize()
    for a, b in zip(sel, (t.cand_job, t.cand_cut, t.cand_score)):
        assert torch.equal(a, b)


def test_stress_hysteresis_full_size(oracle):
    """The hysteresis rule at the full Stress size (the gaps' own capacity set, a gain of one slice):
    sampled pairs and whole sampled rows of the cut matrix, the fused candidates for every gap, and
    every grant's cut and score recomputed by the oracle under the rule."""
    import torch
    import paper_2509_19086_amd as P
    wl = make_workload("stress", 0)
    G, J = wl.n_gaps, wl.n_jobs
    cap_set = np.unique(wl.C).astype(np.int32)
    min_gain = int(cap_set[0])
    eng = P.Engine(0)
    eng.sja_set_hysteresis(cap_set, min_gain)
    t = P.DeviceTick(eng, wl, want_bits=True)
    par = P.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override, 8)
    opar = oracle.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override, 8)
    t.prepare(); t.fit(); t.select(par)
    torch.cuda.synchronize()

    rng = np.random.default_rng(47)
    gi = rng.integers(0, G, size=300_000).astype(np.int32)
    ji = rng.integers(0, J, size=300_000).astype(np.int32)
    want, _, _ = oracle.fit_pairs_hysteresis(gi, ji, wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, wl.W, wl.C,
                                             cap_set, min_gain)
    plain, _, _ = oracle.fit_pairs(gi, ji, wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, wl.W, wl.C)
    assert (want != plain).mean() > 0.05                       # the rule acts
    flat = torch.from_numpy(gi.astype(np.int64) * J + ji.astype(np.int64)).cuda()
    np.testing.assert_array_equal(t.cut.view(-1)[flat].cpu().numpy(), want)

    rows = np.unique(np.concatenate([[0, G - 1, int(np.argmax(wl.W))], rng.integers(0, G, size=8)])).astype(np.int64)
    cut_r, bits_r = oracle.fit_hysteresis(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress,
                                          np.ascontiguousarray(wl.W[rows]), np.ascontiguousarray(wl.C[rows]),
                                          cap_set, min_gain, want_bits=True)
    rows_t = torch.from_numpy(rows).cuda()
    np.testing.assert_array_equal(t.cut[rows_t].cpu().numpy(), cut_r)
    np.testing.assert_array_equal(t.bits[rows_t].cpu().numpy().view(np.uint32), bits_r)
    pd, pp, _ = oracle.prepare(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress)
    cj, cc, cs = oracle.select(cut_r, wl.seg_off, pd, pp, opar, wl.wait, wl.sla_class)
    np.testing.assert_array_equal(t.cand_job[rows_t].cpu().numpy(), cj)
    np.testing.assert_array_equal(t.cand_cut[rows_t].cpu().numpy(), cc)
    np.testing.assert_array_equal(t.cand_score[rows_t].cpu().numpy(), cs)

    sel = (t.cand_job.clone(), t.cand_cut.clone(), t.cand_score.clone())
    t.fit_select(par)
    torch.cuda.synchronize()
    for a, b in zip(sel, (t.cand_job, t.cand_cut, t.cand_score)):
        assert torch.equal(a, b)

    t.resolve(par)
    gj = t.grant_job.cpu().numpy(); gc = t.grant_cut.cpu().numpy(); gs = t.grant_score.cpu().numpy()
    jg = t.job_gap.cpu().numpy()
    granted = np.nonzero(gj >= 0)[0]
    assert len(granted) > 500 and len(np.unique(gj[granted])) == len(granted)
    np.testing.assert_array_equal(jg[gj[granted]], granted)
    ocut, sd, sp = oracle.fit_pairs_hysteresis(granted.astype(np.int32), gj[granted], wl.seg_off, wl.dur, wl.mem,
                                               wl.safe, wl.progress, wl.W, wl.C, cap_set, min_gain)
    np.testing.assert_array_equal(gc[granted], ocut)
    np.testing.assert_array_equal(gs[granted], sd * sp * (wl.wait_scale + wl.wait[gj[granted]].astype(np.int64)))
    assert gj[0] == cj[0] and gc[0] == cc[0] and gs[0] == cs[0]
    eng.sja_set_hysteresis(None)
