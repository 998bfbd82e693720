"""sja_validate on the GPU: the generated workloads pass, and each planted violation of a
precondition is reported with its own bit (the violations are planted in the inputs on the host;
every kernel involved stays inside its arrays)."""
import numpy as np
import pytest

from gen import make_workload

pytestmark = pytest.mark.gpu

OFFSETS, DURATION, MEMORY, PROGRESS, DURATION_SUM, CLASS, WAIT, SCORE = 1, 2, 4, 8, 16, 32, 64, 128


@pytest.fixture(scope="module")
def engine():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2509_19086_amd as P
    return P.Engine(0)


def _run(engine, seg_off, dur, mem, progress, params=None, wait=None, cls=None):
    import torch
    up = lambda a, dt: None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=dt)).cuda()
    out = torch.full((1,), -1, dtype=torch.int32, device="cuda:0")
    engine.sja_validate(up(seg_off, np.int64), up(dur, np.int32), up(mem, np.int32), up(progress, np.int32),
                        params, up(wait, np.int32), up(cls, np.uint8), out)
    return int(out.item()) & 0xffffffff


@pytest.mark.parametrize("name", ["tiny", "small", "medium"])
def test_generated_workloads_pass(engine, name):
    import paper_2509_19086_amd as P
    wl = make_workload(name, 0)
    assert _run(engine, wl.seg_off, wl.dur, wl.mem, wl.progress) == 0
    for policy in range(4):
        par = P.Params.make(policy, wl.wait_scale, wl.sla_weight, wl.class0_override, 0)
        assert _run(engine, wl.seg_off, wl.dur, wl.mem, wl.progress, par, wl.wait, wl.sla_class) == 0


def test_stress_passes(engine):
    import paper_2509_19086_amd as P
    wl = make_workload("stress", 0)
    par = P.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override, 0)
    assert _run(engine, wl.seg_off, wl.dur, wl.mem, wl.progress, par, wl.wait, wl.sla_class) == 0


def test_each_violation_has_its_bit(engine):
    import paper_2509_19086_amd as P
    wl = make_workload("small", 1, n_gaps=8, n_jobs=300)
    S, J = wl.n_segments, wl.n_jobs
    base = dict(seg_off=wl.seg_off.copy(), dur=wl.dur.copy(), mem=wl.mem.copy(), progress=wl.progress.copy())
    par = P.Params.make(3, wl.wait_scale, wl.sla_weight, wl.class0_override, 0)

    def run(params=None, wait=None, cls=None, **change):
        a = {k: v.copy() for k, v in base.items()}
        for k, (i, v) in change.items():
            a[k][i] = v
        return _run(engine, a["seg_off"], a["dur"], a["mem"], a["progress"], params, wait, cls)

    assert run() == 0
    assert run(seg_off=(0, 1)) == OFFSETS                                  # does not start at 0
    assert run(seg_off=(J, S - 1)) == OFFSETS                              # does not end at n_segments
    assert run(seg_off=(J, S + 7)) == OFFSETS                              # ends beyond the arrays
    assert run(seg_off=(5, int(wl.seg_off[7]) + 1)) & OFFSETS              # decreases between jobs 5 and 6..7
    assert run(seg_off=(9, -4)) & OFFSETS
    assert run(dur=(S // 2, 0)) == DURATION
    assert run(dur=(S - 1, -3)) == DURATION
    assert run(mem=(0, -1)) == MEMORY
    assert run(progress=(17, -1)) == PROGRESS
    L17 = int(wl.seg_off[18] - wl.seg_off[17])
    assert run(progress=(17, L17)) == 0                                    # finished is fine
    assert run(progress=(17, L17 + 1)) == PROGRESS
    assert run(dur=(S // 3, 2**31 - 1)) == DURATION_SUM                    # one huge segment pushes the job's sum over
    assert run(dur=(S // 2, 0), mem=(3, -9), progress=(0, -5)) == DURATION | MEMORY | PROGRESS
    # policy inputs
    cls = wl.sla_class.copy(); cls[40] = 3
    assert run(par, wl.wait, cls) == CLASS
    assert run(P.Params.make(1, wl.wait_scale, wl.sla_weight, 1, 0), wl.wait, cls) == 0    # FAIRNESS never reads the class
    wait = wl.wait.copy(); wait[41] = -2
    assert run(par, wait, wl.sla_class) == WAIT
    assert run(P.Params.make(2, wl.wait_scale, wl.sla_weight, 1, 0), wait, wl.sla_class) == 0  # SLA never reads the wait
    # score range: duration sum ~1.3e4 x memory 40960 x (1000 + wait) stays far below 2^62 ...
    assert run(par, wl.wait, wl.sla_class) == 0
    # ... until one job's memory and wait are pushed to the top of int32
    big_wait = wl.wait.copy(); big_wait[7] = 2**31 - 1 - wl.wait_scale
    k7 = int(wl.seg_off[7])
    assert run(par, big_wait, wl.sla_class, mem=(k7, 2**31 - 1)) == SCORE
    assert run(P.Params.make(0), None, None, mem=(k7, 2**31 - 1)) == 0     # EFFICIENCY: F alone fits


def test_validate_argument_checks(engine):
    import torch
    import paper_2509_19086_amd as P
    wl = make_workload("tiny", 0)
    with pytest.raises(RuntimeError):                                      # FAIRNESS needs the waits
        _run(engine, wl.seg_off, wl.dur, wl.mem, wl.progress, P.Params.make(1), None, None)
    with pytest.raises(RuntimeError):
        _run(engine, wl.seg_off, wl.dur, wl.mem, wl.progress, P.Params.make(9), wl.wait, wl.sla_class)
    # empty job table
    assert _run(engine, np.zeros(1, np.int64), np.zeros(0, np.int32), np.zeros(0, np.int32), np.zeros(0, np.int32)) == 0
