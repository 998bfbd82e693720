"""GPU parity at the full sizes of Large and Stress, element by element.

Every entry of the cut matrix, every interest word and every gap's candidate
(job, cut, score) is compared with the oracle's, nothing summed or sampled:
the oracle evaluates the same gaps a block of 256 rows at a time, and each
block is compared with the library's rows for those gaps with
assert_array_equal.  The library runs once per config on the whole batch (the
launch configuration bench.py times); the comparison is cut into slices of gaps
so that no single test is quiet for minutes.  The fused call's candidates are
compared for every gap as well.
"""
import numpy as np
import pytest

from gen import make_workload

pytestmark = [pytest.mark.gpu, pytest.mark.slow]

BLOCK = 256
SLICES = {"large": 2, "stress": 8}


class _Run:
    """One whole-batch tick on the GPU plus what the oracle needs to follow it."""

    def __init__(self, oracle, name):
        import torch
        import paper_2509_19086_amd as P
        self.wl = wl = make_workload(name, 0)
        self.eng = P.Engine(0)
        self.t = t = P.DeviceTick(self.eng, wl, want_bits=True)
        self.par = P.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override, 0)
        self.opar = oracle.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override, 0)
        t.prepare(); t.fit(); t.select(self.par)
        torch.cuda.synchronize()
        self.sel = tuple(x.cpu().numpy().copy() for x in (t.cand_job, t.cand_cut, t.cand_score))
        for out in (t.cand_job, t.cand_cut, t.cand_score):
            out.fill_(-5)
        t.fit_select(self.par)
        torch.cuda.synchronize()
        self.fused = tuple(x.cpu().numpy().copy() for x in (t.cand_job, t.cand_cut, t.cand_score))
        self.pd, self.pp, self.ps = oracle.prepare(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress)


@pytest.fixture(scope="module")
def runs(oracle):
    cache = {}

    def get(name):
        if name not in cache:
            cache.clear()                       # one config's matrix on the GPU at a time
            cache[name] = _Run(oracle, name)
        return cache[name]
    yield get
    cache.clear()


def _cases():
    return [(name, k) for name in ("large", "stress") for k in range(SLICES[name])]


@pytest.mark.parametrize("name,part", _cases())
def test_every_element_of_fit_and_select(oracle, runs, name, part):
    r = runs(name)
    wl, t = r.wl, r.t
    G = wl.n_gaps
    per = (G + SLICES[name] - 1) // SLICES[name]
    lo, hi = part * per, min(G, (part + 1) * per)
    if part == 0:
        np.testing.assert_array_equal(t.pre_dur.cpu().numpy().astype(np.int64), r.pd)
        np.testing.assert_array_equal(t.pre_peak.cpu().numpy().astype(np.int64), r.pp)
        np.testing.assert_array_equal(t.prev_safe.cpu().numpy(), r.ps)
    for g0 in range(lo, hi, BLOCK):
        g1 = min(hi, g0 + BLOCK)
        W = np.ascontiguousarray(wl.W[g0:g1])
        C = np.ascontiguousarray(wl.C[g0:g1])
        cut, bits = oracle.fit(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, W, C)
        cj, cc, cs = oracle.select(cut, wl.seg_off, r.pd, r.pp, r.opar, wl.wait, wl.sla_class)
        where = f"{name}: gaps {g0}..{g1 - 1}"
        np.testing.assert_array_equal(t.cut[g0:g1].cpu().numpy(), cut, err_msg=where)
        np.testing.assert_array_equal(t.bits[g0:g1].cpu().numpy().view(np.uint32), bits, err_msg=where)
        for got, fused, want in zip(r.sel, r.fused, (cj, cc, cs)):
            np.testing.assert_array_equal(got[g0:g1], want, err_msg=where)
            np.testing.assert_array_equal(fused[g0:g1], want, err_msg=where + " (fused call)")
