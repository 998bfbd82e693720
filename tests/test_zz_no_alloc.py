"""The entry point for callers that cannot allocate, sja_prepare_profiles_static, through the
C ABI against sja_prepare_profiles: the running tables it returns, and - because the private
tables it leaves in the library's built-in scratch are what the rest of the tick reads - the
cut matrix, the interest rows, the candidates and the grants of the calls that follow, all
bit for bit.  Two ticks in a row on the same scratch, the second with a smaller input, so that
whatever the first left behind must not leak into the second."""
import ctypes

import numpy as np
import pytest

from gen import make_workload

pytestmark = pytest.mark.gpu


def _tick(P, eng, wl, static):
    """One whole tick through the engine's own methods; returns every output as numpy."""
    import torch
    dev = "cuda:0"
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    G, J, S = wl.n_gaps, wl.n_jobs, int(wl.seg_off[-1])
    seg_off, dur, mem, safe, progress = up(wl.seg_off), up(wl.dur), up(wl.mem), up(wl.safe), up(wl.progress)
    W, C, wait, cls = up(wl.W), up(wl.C), up(wl.wait), up(wl.sla_class)
    i32 = dict(dtype=torch.int32, device=dev)
    pre_dur, pre_peak, prev_safe = (torch.full((S,), -7, **i32) for _ in range(3))
    cut = torch.full((G, J), -9, **i32)
    bits = torch.full((G, (J + 31) // 32), -9, **i32)
    cand = [torch.full((G,), -9, **i32), torch.full((G,), -9, **i32),
            torch.full((G,), -9, dtype=torch.int64, device=dev)]
    grant = [torch.full((G,), -9, **i32), torch.full((G,), -9, **i32),
             torch.full((G,), -9, dtype=torch.int64, device=dev)]
    job_gap = torch.full((J,), -9, **i32)
    rounds = torch.zeros(2, **i32)
    par = P.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override, wl.max_rounds)
    prepare = eng.sja_prepare_profiles_static if static else eng.sja_prepare_profiles
    prepare(seg_off, dur, mem, safe, progress, pre_dur, pre_peak, prev_safe)
    eng.sja_fit(W, C, cut, bits)
    eng.sja_select(par, wait, cls, None, None, *cand)
    eng.sja_resolve(par, wait, cls, *grant, job_gap, rounds)
    torch.cuda.synchronize()
    outs = [pre_dur, pre_peak, prev_safe, cut, bits, *cand, *grant, job_gap, rounds]
    return [o.cpu().numpy() for o in outs]


def test_static_scratch_prepare_matches_the_workspace_one():
    import torch
    import paper_2509_19086_amd as P
    assert torch.cuda.is_available(), "this test needs the GPU"
    lib = P.load_library()
    limit = 64 << 20
    first = make_workload("small", 2, n_gaps=200, n_jobs=700)
    second = make_workload("medium", 5, n_gaps=96, n_jobs=150)           # smaller in every dimension
    assert second.n_jobs < first.n_jobs and int(second.seg_off[-1]) < int(first.seg_off[-1])
    for wl in (first, second):
        assert 0 < lib.sja_workspace_bytes(wl.n_gaps, wl.n_jobs, int(wl.seg_off[-1])) <= limit

    # the reference: the existing entry point on a caller-owned workspace
    ref_eng = P.Engine(0)
    want = []
    for wl in (first, second):
        ref_eng.ensure_workspace(wl.n_gaps, wl.n_jobs, int(wl.seg_off[-1]))
        want.append(_tick(P, ref_eng, wl, static=False))

    # the new entry point: no workspace is ever handed to this context
    eng = P.Engine(0)
    assert eng.workspace is None
    for wl, ref in zip((first, second), want):
        got = _tick(P, eng, wl, static=True)
        assert eng.workspace is None
        for k, (a, b) in enumerate(zip(got, ref)):
            np.testing.assert_array_equal(a, b, err_msg=f"output {k}, {wl.n_gaps} gaps x {wl.n_jobs} jobs")
        assert (got[3] >= 0).any() and (got[8] >= 0).any()              # the tick did something

    # sizes beyond the built-in scratch are refused on the host, with the reason
    vp = ctypes.c_void_p
    junk = vp(256)
    rc = lib.sja_prepare_profiles_static(eng.h, None, 1 << 20, 1 << 28, junk, junk, junk, junk, junk, junk, junk, junk)
    assert rc == -2 and b"built-in scratch" in lib.sja_last_error(eng.h)
