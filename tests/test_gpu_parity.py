"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle.

Everything is integer work, so the bar is bit-exact equality, element by
element, on the same seeded inputs.
"""
import numpy as np
import pytest

from gen import make_workload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def engine():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2509_19086_amd as P
    return P.Engine(0)


def _params(P, wl, max_rounds=None):
    return P.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override,
                         wl.max_rounds if max_rounds is None else max_rounds)


def _oracle_params(O, wl, policy=None, max_rounds=None):
    return O.Params.make(wl.policy if policy is None else policy, wl.wait_scale, wl.sla_weight,
                         wl.class0_override, wl.max_rounds if max_rounds is None else max_rounds)


def full_tick_check(engine, oracle, wl, policies=None, check_resolve=True, resolve_modes=(0, 1, 2)):
    """prepare, fit, select (each policy), resolve: every output equals the oracle's.
    Resolve runs once per mode (candidate lists / matrix-scanning rounds): each
    must reproduce the oracle's rounds exactly."""
    import torch
    import paper_2509_19086_amd as P
    t = P.DeviceTick(engine, wl)
    t.prepare()
    t.fit()
    torch.cuda.synchronize()

    pd, pp, ps = oracle.prepare(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress)
    np.testing.assert_array_equal(t.pre_dur.cpu().numpy().astype(np.int64), pd)
    np.testing.assert_array_equal(t.pre_peak.cpu().numpy().astype(np.int64), pp)
    np.testing.assert_array_equal(t.prev_safe.cpu().numpy(), ps)

    cut, bits = oracle.fit(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, wl.W, wl.C)
    np.testing.assert_array_equal(t.cut.cpu().numpy(), cut)
    np.testing.assert_array_equal(t.bits.cpu().numpy().view(np.uint32), bits)

    for policy in (policies if policies is not None else [wl.policy]):
        par = P.Params.make(policy, wl.wait_scale, wl.sla_weight, wl.class0_override, wl.max_rounds)
        t.select(par)
        torch.cuda.synchronize()
        cj, cc, cs = oracle.select(cut, wl.seg_off, pd, pp, _oracle_params(oracle, wl, policy),
                                   wl.wait, wl.sla_class)
        np.testing.assert_array_equal(t.cand_job.cpu().numpy(), cj)
        np.testing.assert_array_equal(t.cand_cut.cpu().numpy(), cc)
        np.testing.assert_array_equal(t.cand_score.cpu().numpy(), cs)
        if check_resolve:
            gj, gc, gs, jg, rounds, stable = oracle.resolve(
                cut, wl.seg_off, pd, pp, _oracle_params(oracle, wl, policy), wl.wait, wl.sla_class)
            try:
                for mode in resolve_modes:
                    engine.sja_set_resolve_mode(mode)
                    for out in (t.grant_job, t.grant_cut, t.grant_score, t.job_gap, t.rounds):
                        out.fill_(-5)
                    t.resolve(par)
                    np.testing.assert_array_equal(t.grant_job.cpu().numpy(), gj, err_msg=f"mode {mode}")
                    np.testing.assert_array_equal(t.grant_cut.cpu().numpy(), gc, err_msg=f"mode {mode}")
                    np.testing.assert_array_equal(t.grant_score.cpu().numpy(), gs, err_msg=f"mode {mode}")
                    np.testing.assert_array_equal(t.job_gap.cpu().numpy(), jg, err_msg=f"mode {mode}")
                    assert t.rounds.cpu().tolist() == [rounds, stable], f"mode {mode}"
            finally:
                engine.sja_set_resolve_mode(0)
    return t


@pytest.mark.parametrize("seed", [0, 1, 2, 3, 4])
def test_tiny_all_policies(engine, oracle, seed):
    full_tick_check(engine, oracle, make_workload("tiny", seed), policies=[0, 1, 2, 3])


@pytest.mark.parametrize("seed", [0, 1, 2, 3, 4])
def test_small_all_policies(engine, oracle, seed):
    full_tick_check(engine, oracle, make_workload("small", seed), policies=[1, 0, 2, 3])


@pytest.mark.parametrize("seed", [0, 1, 2, 3, 4])
def test_medium(engine, oracle, seed):
    full_tick_check(engine, oracle, make_workload("medium", seed))


@pytest.mark.parametrize("name,G,J", [("large", 300, 1000), ("stress", 777, 2500),
                                      ("stress", 130, 70), ("medium", 1, 1), ("small", 257, 65)])
def test_ragged_shapes(engine, oracle, name, G, J):
    """Sizes that are no multiple of any tile: ragged job tiles, gap chunks, bit words."""
    wl = make_workload(name, 7, n_gaps=G, n_jobs=J)
    full_tick_check(engine, oracle, wl, policies=[wl.policy, 3])


@pytest.mark.parametrize("n_classes", [1, 63, 64, 65, 700])
def test_many_capacity_classes(engine, oracle, n_classes):
    """Few distinct capacities take the table-driven fit path, many the searching one."""
    wl = make_workload("medium", 11, n_gaps=700, n_jobs=900)
    rng = np.random.default_rng(n_classes)
    caps = np.sort(rng.choice(np.arange(300, 90000), size=n_classes, replace=False)).astype(np.int32)
    wl.C = np.ascontiguousarray(caps[rng.integers(0, n_classes, size=wl.n_gaps)])
    if n_classes == 700:
        wl.C = np.ascontiguousarray(rng.permutation(caps))          # every gap its own capacity
    full_tick_check(engine, oracle, wl, policies=[2, 3])


def test_round_cap(engine, oracle):
    wl = make_workload("small", 3)
    for cap in (1, 2, 8):
        wl.max_rounds = cap
        full_tick_check(engine, oracle, wl, policies=[0])


@pytest.mark.parametrize("cap", [0, 64, 191, 192, 400])
def test_long_chain_of_rounds(engine, oracle, cap):
    """Hundreds of rounds: gaps that all want the same jobs are granted one per round, so the
    resolve runs through several batches of round launches; caps inside a batch and at the
    edges of one."""
    wl = make_workload("small", 11, n_gaps=700, n_jobs=1200)
    wl.W = np.full_like(wl.W, 1500)
    wl.W[::7] += np.arange(len(wl.W[::7]), dtype=wl.W.dtype)          # a few gaps differ a little
    wl.C = np.full_like(wl.C, 40960)
    wl.max_rounds = cap
    t = full_tick_check(engine, oracle, wl, policies=[0, 3], resolve_modes=(0,))
    if cap == 0:
        assert t.rounds.cpu().tolist()[0] > 448                        # past the third batch (64 + 128 + 256)


def test_select_with_held_jobs_and_inactive_gaps(engine, oracle):
    import torch
    import paper_2509_19086_amd as P
    wl = make_workload("small", 5)
    t = P.DeviceTick(engine, wl)
    t.prepare()
    t.fit()
    rng = np.random.default_rng(0)
    held = np.where(rng.random(wl.n_jobs) < 0.5, 3, -1).astype(np.int32)
    act = (rng.random(wl.n_gaps) < 0.7).astype(np.uint8)
    pd, pp, _ = oracle.prepare(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress)
    cut, _ = oracle.fit(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, wl.W, wl.C, False)
    for policy in (0, 1, 2, 3):
        par = P.Params.make(policy)
        t.select(par, torch.from_numpy(held).cuda(), torch.from_numpy(act).cuda())
        torch.cuda.synchronize()
        cj, cc, cs = oracle.select(cut, wl.seg_off, pd, pp, oracle.Params.make(policy), wl.wait,
                                   wl.sla_class, held, act)
        np.testing.assert_array_equal(t.cand_job.cpu().numpy(), cj)
        np.testing.assert_array_equal(t.cand_cut.cpu().numpy(), cc)
        np.testing.assert_array_equal(t.cand_score.cpu().numpy(), cs)


def test_degenerate_profiles(engine, oracle):
    """Empty jobs, finished jobs, monoliths, all-safe jobs, W/C at the int32 limits."""
    import types
    rng = np.random.default_rng(1)
    lens = np.array([0, 5, 1, 0, 64, 65, 128, 3, 200, 0], dtype=np.int64)
    seg_off = np.zeros(len(lens) + 1, dtype=np.int64)
    np.cumsum(lens, out=seg_off[1:])
    S = int(seg_off[-1])
    dur = rng.integers(1, 50, size=S).astype(np.int32)
    mem = rng.integers(0, 1000, size=S).astype(np.int32)
    safe = (rng.random(S) < 0.3).astype(np.uint8)
    safe[seg_off[4]:seg_off[5]] = 0                    # monolith
    safe[seg_off[5]:seg_off[6]] = 1                    # every boundary safe
    progress = np.array([0, 5, 0, 0, 0, 64, 127, 1, 77, 0], dtype=np.int32)  # job 1 finished
    W = np.array([2**31 - 1, 0, 1, 100, 5000, 2**31 - 1, 300, -5], dtype=np.int32)
    C = np.array([2**31 - 1, 500, 999, 0, 700, 400, 2**31 - 1, 900], dtype=np.int32)
    wl = types.SimpleNamespace(
        seg_off=seg_off, dur=dur, mem=mem, safe=safe, progress=progress, W=W, C=C,
        wait=rng.integers(0, 100, size=len(lens)).astype(np.int32),
        sla_class=rng.integers(0, 3, size=len(lens)).astype(np.uint8),
        policy=3, wait_scale=1000, sla_weight=(4, 2, 1), class0_override=1, max_rounds=0,
        n_gaps=len(W), n_jobs=len(lens))
    full_tick_check(engine, oracle, wl, policies=[0, 1, 2, 3])


def test_empty_batches(engine):
    import torch
    import paper_2509_19086_amd as P
    wl = make_workload("tiny", 0, n_gaps=0, n_jobs=4)
    t = P.DeviceTick(engine, wl)
    t.prepare(); t.fit(); t.select(P.Params.make(0)); t.resolve(P.Params.make(0))
    torch.cuda.synchronize()
    assert t.rounds.cpu().tolist() == [1, 1] and (t.job_gap.cpu().numpy() == -1).all()


def test_repeatable(engine):
    """Three runs of the whole tick give byte-identical outputs (atomics included)."""
    import torch
    import paper_2509_19086_amd as P
    wl = make_workload("small", 9)
    outs = []
    for _ in range(3):
        t = P.DeviceTick(engine, wl)
        t.prepare(); t.fit(); t.select(P.Params.make(3)); t.resolve(P.Params.make(3))
        torch.cuda.synchronize()
        outs.append([x.cpu().numpy().tobytes() for x in
                     (t.cut, t.bits, t.cand_job, t.cand_score, t.grant_job, t.grant_score, t.job_gap, t.rounds)])
    assert outs[0] == outs[1] == outs[2]


def fused_check(engine, oracle, wl, policies, held=None, act=None, resolve=True):
    """sja_fit_select reports what sja_select reports after sja_fit (the oracle's), and
    sja_resolve works on top of it without any cut matrix."""
    import torch
    import paper_2509_19086_amd as P
    t = P.DeviceTick(engine, wl, want_cut=False)
    t.prepare()
    pd, pp, _ = oracle.prepare(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress)
    cut, _ = oracle.fit(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, wl.W, wl.C, False)
    h = None if held is None else torch.from_numpy(held).cuda()
    a = None if act is None else torch.from_numpy(act).cuda()
    for policy in policies:
        par = P.Params.make(policy, wl.wait_scale, wl.sla_weight, wl.class0_override, wl.max_rounds)
        opar = _oracle_params(oracle, wl, policy)
        for out in (t.cand_job, t.cand_cut, t.cand_score):
            out.fill_(-5)
        t.fit_select(par, h, a)
        torch.cuda.synchronize()
        cj, cc, cs = oracle.select(cut, wl.seg_off, pd, pp, opar, wl.wait, wl.sla_class, held, act)
        np.testing.assert_array_equal(t.cand_job.cpu().numpy(), cj, err_msg=f"policy {policy}")
        np.testing.assert_array_equal(t.cand_cut.cpu().numpy(), cc, err_msg=f"policy {policy}")
        np.testing.assert_array_equal(t.cand_score.cpu().numpy(), cs, err_msg=f"policy {policy}")
        if resolve and held is None and act is None:
            t.resolve(par)
            gj, gc, gs, jg, rounds, stable = oracle.resolve(cut, wl.seg_off, pd, pp, opar, wl.wait, wl.sla_class)
            np.testing.assert_array_equal(t.grant_job.cpu().numpy(), gj)
            np.testing.assert_array_equal(t.grant_cut.cpu().numpy(), gc)
            np.testing.assert_array_equal(t.grant_score.cpu().numpy(), gs)
            np.testing.assert_array_equal(t.job_gap.cpu().numpy(), jg)
            assert t.rounds.cpu().tolist() == [rounds, stable]
    return t


@pytest.mark.parametrize("name,seed", [("tiny", 0), ("tiny", 3), ("small", 0), ("small", 2), ("medium", 0)])
def test_fused_fit_select(engine, oracle, name, seed):
    fused_check(engine, oracle, make_workload(name, seed), policies=[0, 1, 2, 3])


@pytest.mark.parametrize("name,G,J", [("large", 300, 1000), ("stress", 777, 2500),
                                      ("stress", 130, 70), ("medium", 1, 1), ("small", 257, 65)])
def test_fused_ragged_shapes(engine, oracle, name, G, J):
    wl = make_workload(name, 7, n_gaps=G, n_jobs=J)
    fused_check(engine, oracle, wl, policies=[wl.policy, 3])


def test_fused_with_held_jobs_and_inactive_gaps(engine, oracle):
    wl = make_workload("small", 5)
    rng = np.random.default_rng(0)
    held = np.where(rng.random(wl.n_jobs) < 0.5, 3, -1).astype(np.int32)
    act = (rng.random(wl.n_gaps) < 0.7).astype(np.uint8)
    fused_check(engine, oracle, wl, policies=[0, 1, 2, 3], held=held, act=act)


@pytest.mark.parametrize("n_classes", [1, 64, 65, 700])
def test_fused_many_capacity_classes(engine, oracle, n_classes):
    """Beyond 64 capacities the stepping kernel searches for itself; the candidates stay the same.
    (There sja_resolve would need the matrix-scanning rounds, so only the candidates are checked.)"""
    wl = make_workload("small", 9, n_gaps=900, n_jobs=700)
    rng = np.random.default_rng(n_classes)
    caps = np.sort(rng.choice(np.arange(2000, 60000), size=n_classes, replace=False)).astype(np.int32)
    wl.C = caps[rng.integers(0, n_classes, size=wl.n_gaps)].astype(np.int32)
    fused_check(engine, oracle, wl, policies=[3, 0], resolve=True)


def test_fused_then_select_is_refused_and_scanning_rounds_work(engine, oracle):
    """After sja_fit_select there is no matrix: sja_select is refused, while the scanning rounds
    re-evaluate the pairs and give the oracle's grants."""
    import torch
    import paper_2509_19086_amd as P
    wl = make_workload("tiny", 0)
    t = P.DeviceTick(engine, wl, want_cut=False)
    t.prepare()
    par = P.Params.make(0)
    t.fit_select(par)
    pd, pp, _ = oracle.prepare(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress)
    cut, _ = oracle.fit(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, wl.W, wl.C, False)
    want = oracle.resolve(cut, wl.seg_off, pd, pp, oracle.Params.make(0), wl.wait, wl.sla_class)
    try:
        engine.sja_set_resolve_mode(1)
        t.resolve(par)
        for got, exp in zip((t.grant_job, t.grant_cut, t.grant_score, t.job_gap), want[:4]):
            np.testing.assert_array_equal(got.cpu().numpy(), exp)
        assert t.rounds.cpu().tolist() == [want[4], want[5]]
        with pytest.raises(P.SjaError):
            t.select(par)
    finally:
        engine.sja_set_resolve_mode(0)
    torch.cuda.synchronize()


def test_random_small_shapes(engine, oracle):
    """Sixty random shapes from one gap x one job to 130 x 400, every generator, every policy:
    the whole tick in both resolve modes, and the fused call with resolve on top of it."""
    rng = np.random.default_rng(20240)
    names = ["tiny", "small", "medium", "large", "stress"]
    for case in range(60):
        name = names[case % len(names)]
        G = int(rng.integers(1, 131))
        J = int(rng.integers(1, 401))
        if case % 7 == 0:
            G, J = (1, J) if case % 14 == 0 else (G, 1)
        wl = make_workload(name, 100 + case, n_gaps=G, n_jobs=J)
        if case % 5 == 0:                                   # windows and capacities from zero up: many declines
            wl.W = np.ascontiguousarray((wl.W * rng.random(G)).astype(np.int32))
            wl.C = np.ascontiguousarray((wl.C * rng.random(G)).astype(np.int32))
        policy = int(rng.integers(0, 4))
        wl.max_rounds = int(rng.integers(0, 4)) if case % 3 == 0 else 0
        full_tick_check(engine, oracle, wl, policies=[policy])
        # with more than 64 distinct capacities the rounds scan the matrix, which the fused call never writes
        fused_check(engine, oracle, wl, [policy], resolve=len(np.unique(wl.C)) <= 64)


def test_more_jobs_than_the_held_bitmap_holds(engine, oracle):
    """With more than 131072 jobs the early rounds cannot keep the held jobs as a bitmap in LDS and
    walk by claim words from the first round on: same grants."""
    wl = make_workload("tiny", 5, n_gaps=96, n_jobs=140000)
    full_tick_check(engine, oracle, wl, policies=[wl.policy, 3], resolve_modes=(0,))


@pytest.mark.parametrize("policy", [0, 3])
def test_resolve_after_the_fused_call_with_too_many_capacities(engine, oracle, policy):
    """After sja_fit_select there is no cut matrix, and with more than 64 distinct capacities the
    candidate lists cannot run either: the rounds then re-evaluate the pairs of the still-active
    gaps each round.  Same grants as the oracle's, in both resolve modes, also under a round cap."""
    import paper_2509_19086_amd as P
    wl = make_workload("medium", 13, n_gaps=300, n_jobs=200)
    wl.C = np.ascontiguousarray((9000 + 7 * np.arange(wl.n_gaps)).astype(np.int32))     # 300 distinct capacities
    t = P.DeviceTick(engine, wl, want_cut=False)
    pd, pp, _ = oracle.prepare(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress)
    cut, _ = oracle.fit(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, wl.W, wl.C, False)
    t.prepare()
    for cap in (0, 3):
        par = P.Params.make(policy, wl.wait_scale, wl.sla_weight, wl.class0_override, cap)
        opar = oracle.Params.make(policy, wl.wait_scale, wl.sla_weight, wl.class0_override, cap)
        want = oracle.resolve(cut, wl.seg_off, pd, pp, opar, wl.wait, wl.sla_class)
        assert want[4] > 3 or cap == 3
        try:
            for mode in (0, 1):
                engine.sja_set_resolve_mode(mode)
                t.fit_select(par)
                for o in (t.grant_job, t.grant_cut, t.grant_score, t.job_gap, t.rounds):
                    o.fill_(-5)
                t.resolve(par)
                for got, exp in zip((t.grant_job, t.grant_cut, t.grant_score, t.job_gap), want[:4]):
                    np.testing.assert_array_equal(got.cpu().numpy(), exp, err_msg=f"cap {cap} mode {mode}")
                assert t.rounds.cpu().tolist() == [want[4], want[5]]
        finally:
            engine.sja_set_resolve_mode(0)


def test_largest_gap_count(engine, oracle):
    """The advertised maximum of 2^20 gaps with a handful of jobs (two capacity classes, ragged
    job count): every output of the tick against the oracle, both kinds of rounds."""
    wl = make_workload("small", 21, n_gaps=1 << 20, n_jobs=37)
    wl.C = np.ascontiguousarray(np.where(np.arange(wl.n_gaps) % 3 == 0, 20480, 40960).astype(np.int32))
    full_tick_check(engine, oracle, wl, policies=[wl.policy])


def test_store_reference_writes_the_whole_matrix(engine):
    """The measurement aid covers exactly the pair matrix: afterwards cut[g][j] = j for every pair
    (ragged sizes, several capacity classes), and it refuses to run without a plan."""
    import torch
    import paper_2509_19086_amd as P
    for name, seed, kw in (("tiny", 0, {}), ("small", 2, {}), ("medium", 3, dict(n_gaps=333, n_jobs=1111))):
        wl = make_workload(name, seed, **kw)
        t = P.DeviceTick(engine, wl, want_bits=False)
        t.prepare()
        with pytest.raises(P.SjaError):
            engine.sja_store_reference(t.cut)
        t.fit()
        t.cut.fill_(-7)
        guard = torch.full((64,), -9, dtype=torch.int32, device="cuda:0")     # allocated right behind: must stay as it is
        engine.sja_store_reference(t.cut)
        torch.cuda.synchronize()
        want = torch.arange(wl.n_jobs, dtype=torch.int32, device="cuda:0").expand(wl.n_gaps, wl.n_jobs)
        assert torch.equal(t.cut.view(wl.n_gaps, wl.n_jobs), want)
        assert bool((guard == -9).all())
        with pytest.raises(P.SjaError):                    # the matrix no longer holds the replies
            t.select(P.Params.make(0))
