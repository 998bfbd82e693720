"""Pins for the CPU oracle's prepare and fit (no GPU).

Each test checks oracle/sja_oracle.c against something other than itself: a
numpy library routine, a closed form, the from-scratch brute force, or an
invariant the paper fixes (a granted subjob fits its window and its slice,
Sec. 3.4 / 3.8 / 3.9; subjobs end at subjob boundaries, Sec. 3.7; longer
fragments are preferred, Sec. 3.9).
"""
import json
import os

import numpy as np
import pytest

from gen import make_workload
from oracle import brute
from helpers import random_gaps, random_jobs

INT_MAX = 2**31 - 1
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _prep(O, w):
    return O.prepare(w.seg_off, w.dur, w.mem, w.safe, w.progress)


# ----------------------------------------------------------------- prepare
@pytest.mark.parametrize("name", ["tiny", "small"])
def test_prepare_matches_numpy_scans(oracle, name):
    w = make_workload(name, 1)
    pd, pp, ps = _prep(oracle, w)
    for j in range(w.n_jobs):
        a, b = int(w.seg_off[j]), int(w.seg_off[j + 1])
        p = int(w.progress[j])
        L = b - a
        assert (pd[a:a + p] == -7).all() and (pp[a:a + p] == -7).all() and (ps[a:a + p] == -7).all()
        np.testing.assert_array_equal(pd[a + p:b], np.cumsum(w.dur[a + p:b].astype(np.int64)))
        np.testing.assert_array_equal(pp[a + p:b], np.maximum.accumulate(w.mem[a + p:b].astype(np.int64)))
        bnd = np.arange(p + 1, L + 1)
        flag = w.safe[a + p:b].astype(np.int64).copy()
        flag[-1] = 1                                   # the end is always safe
        last = np.maximum.accumulate(np.where(flag > 0, bnd, -1))
        np.testing.assert_array_equal(ps[a + p:b], last)


def test_prepare_end_flag_is_ignored(oracle):
    rng = np.random.default_rng(5)
    seg_off, dur, mem, safe, progress = random_jobs(rng, 20, 1, 12, allow_done=False)
    safe0 = safe.copy()
    safe0[seg_off[1:] - 1] = 0
    safe1 = safe.copy()
    safe1[seg_off[1:] - 1] = 1
    r0 = oracle.prepare(seg_off, dur, mem, safe0, progress)
    r1 = oracle.prepare(seg_off, dur, mem, safe1, progress)
    for x, y in zip(r0, r1):
        np.testing.assert_array_equal(x, y)


# --------------------------------------------------------------------- fit
def test_fit_matches_brute_force_on_tiny_random_cases(oracle):
    rng = np.random.default_rng(2024)
    n_pairs = 0
    for case in range(400):
        n_jobs = int(rng.integers(1, 7))
        n_gaps = int(rng.integers(1, 7))
        safe_p = float(rng.choice([0.0, 0.2, 0.5, 1.0]))
        seg_off, dur, mem, safe, progress = random_jobs(rng, n_jobs, 0, 12, safe_p=safe_p)
        W, C = random_gaps(rng, n_gaps, 40, 10)
        if case % 7 == 0:
            W[0] = INT_MAX
        if case % 11 == 0:
            C[-1] = INT_MAX
        cut, bits = oracle.fit(seg_off, dur, mem, safe, progress, W, C)
        ref = np.array(brute.fit_all(seg_off, dur, mem, safe, progress, W, C), dtype=np.int32)
        np.testing.assert_array_equal(cut, ref.reshape(n_gaps, n_jobs))
        for g in range(n_gaps):
            for j in range(n_jobs):
                assert ((int(bits[g, j // 32]) >> (j % 32)) & 1) == int(ref[g][j] >= 0)
        n_pairs += n_gaps * n_jobs
    assert n_pairs > 4000


def test_fit_pairs_agrees_with_fit_and_brute(oracle):
    rng = np.random.default_rng(7)
    seg_off, dur, mem, safe, progress = random_jobs(rng, 9, 1, 14)
    W, C = random_gaps(rng, 8, 50, 10)
    cut, _ = oracle.fit(seg_off, dur, mem, safe, progress, W, C)
    gi, ji = np.meshgrid(np.arange(8), np.arange(9), indexing="ij")
    c2, sd, sp = oracle.fit_pairs(gi.ravel(), ji.ravel(), seg_off, dur, mem, safe, progress, W, C)
    np.testing.assert_array_equal(c2.reshape(8, 9), cut)
    for i, (g, j) in enumerate(zip(gi.ravel(), ji.ravel())):
        if c2[i] >= 0:
            a = int(seg_off[j])
            p = int(progress[j])
            assert sd[i] == int(dur[a + p:a + c2[i]].sum())
            assert sp[i] == int(mem[a + p:a + c2[i]].max())


def _check_invariants(w, cut):
    """Fit by construction, safe ends, maximality, justified declines -- per pair."""
    G, J = cut.shape
    for j in range(J):
        a, b = int(w.seg_off[j]), int(w.seg_off[j + 1])
        p = int(w.progress[j])
        L = b - a
        D = np.cumsum(w.dur[a + p:b].astype(np.int64))        # D[i] <-> boundary p+1+i
        P = np.maximum.accumulate(w.mem[a + p:b].astype(np.int64))
        flag = w.safe[a + p:b].astype(bool).copy()
        if L > p:
            flag[-1] = True
        safe_b = np.nonzero(flag)[0] + p + 1                   # safe boundaries after p
        col = cut[:, j]
        for g in range(G):
            c = int(col[g])
            Wg, Cg = int(w.W[g]), int(w.C[g])
            if c >= 0:
                assert p < c <= L
                assert c == L or w.safe[a + c - 1]
                assert D[c - p - 1] <= Wg and P[c - p - 1] <= Cg
                nxt = safe_b[safe_b > c]
                if len(nxt):
                    n = int(nxt[0])
                    assert D[n - p - 1] > Wg or P[n - p - 1] > Cg
            else:
                if len(safe_b):
                    n = int(safe_b[0])
                    assert D[n - p - 1] > Wg or P[n - p - 1] > Cg


@pytest.mark.parametrize("name,seed", [("tiny", 0), ("tiny", 3), ("small", 0)])
def test_fit_invariants_on_configs(oracle, name, seed):
    w = make_workload(name, seed) if name == "tiny" else make_workload(name, seed, n_gaps=48, n_jobs=160)
    cut, _ = oracle.fit(w.seg_off, w.dur, w.mem, w.safe, w.progress, w.W, w.C)
    _check_invariants(w, cut)
    assert (cut >= 0).any() and (cut < 0).any()


def test_fit_invariants_on_stress_like_csr(oracle):
    w = make_workload("stress", 2, n_gaps=24, n_jobs=96)
    cut, _ = oracle.fit(w.seg_off, w.dur, w.mem, w.safe, w.progress, w.W, w.C)
    _check_invariants(w, cut)


def test_fit_is_monotone_in_window_and_capacity(oracle):
    rng = np.random.default_rng(11)
    w = make_workload("small", 4, n_gaps=64, n_jobs=128)
    cut, _ = oracle.fit(w.seg_off, w.dur, w.mem, w.safe, w.progress, w.W, w.C)
    dW = rng.integers(0, 300, size=w.n_gaps).astype(np.int32)
    dC = rng.integers(0, 9000, size=w.n_gaps).astype(np.int32)
    cut2, _ = oracle.fit(w.seg_off, w.dur, w.mem, w.safe, w.progress, w.W + dW, w.C + dC)
    assert (cut2 >= cut).all()
    assert (cut2 > cut).any()


def test_fit_reduces_to_searchsorted_when_every_boundary_is_safe(oracle):
    rng = np.random.default_rng(3)
    seg_off, dur, mem, safe, progress = random_jobs(rng, 40, 1, 60, d_hi=50, m_hi=1000,
                                                    allow_done=False)
    safe[:] = 1
    G = 32
    W = rng.integers(0, 1500, size=G).astype(np.int32)
    C = np.full(G, INT_MAX, dtype=np.int32)
    cut, _ = oracle.fit(seg_off, dur, mem, safe, progress, W, C)
    for j in range(40):
        a, b = int(seg_off[j]), int(seg_off[j + 1])
        p = int(progress[j])
        D = np.cumsum(dur[a + p:b].astype(np.int64))
        n = np.searchsorted(D, W, side="right")            # boundaries with D <= W
        np.testing.assert_array_equal(cut[:, j], np.where(n > 0, p + n, -1))
    # and the capacity-only case: stop before the first segment with mem > C
    W2 = np.full(G, INT_MAX, dtype=np.int32)
    C2 = rng.integers(0, 1000, size=G).astype(np.int32)
    cut2, _ = oracle.fit(seg_off, dur, mem, safe, progress, W2, C2)
    for j in range(40):
        a, b = int(seg_off[j]), int(seg_off[j + 1])
        p = int(progress[j])
        m = mem[a + p:b]
        for g in range(G):
            over = np.nonzero(m > C2[g])[0]
            n = int(over[0]) if len(over) else len(m)
            assert cut2[g, j] == (p + n if n > 0 else -1)


def test_fit_closed_form_on_constant_profiles(oracle):
    """d = delta, m = mu everywhere; boundary b safe iff (b-p) % s == 0 (or b == L)."""
    rng = np.random.default_rng(17)
    for _ in range(60):
        L = int(rng.integers(1, 40))
        p = int(rng.integers(0, L))
        delta = int(rng.integers(1, 8))
        mu = int(rng.integers(1, 50))
        s = int(rng.integers(1, 7))
        seg_off = np.array([0, L], dtype=np.int64)
        dur = np.full(L, delta, dtype=np.int32)
        mem = np.full(L, mu, dtype=np.int32)
        b = np.arange(1, L + 1)
        safe = (((b - p) % s == 0) & (b > p)).astype(np.uint8)
        G = 24
        W = rng.integers(0, delta * L + 5, size=G).astype(np.int32)
        C = rng.integers(mu - 2, mu + 3, size=G).astype(np.int32)
        cut, _ = oracle.fit(seg_off, dur, mem, safe, np.array([p], dtype=np.int32), W, C)
        for g in range(G):
            n = min(L - p, int(W[g]) // delta)
            if mu > C[g]:
                want = -1
            elif n == L - p:
                want = L
            else:
                want = p + s * (n // s)
                if want == p:
                    want = -1
            assert cut[g, 0] == want, (L, p, delta, mu, s, int(W[g]), int(C[g]))


def test_monolith_is_interested_only_if_its_whole_remainder_fits(oracle):
    """A job without internal subjob boundaries falls back to all-or-nothing (Sec. 4.3)."""
    rng = np.random.default_rng(23)
    seg_off, dur, mem, safe, progress = random_jobs(rng, 30, 1, 20, d_hi=20, m_hi=100,
                                                    allow_done=False)
    safe[:] = 0
    W, C = random_gaps(rng, 40, 250, 110)
    cut, _ = oracle.fit(seg_off, dur, mem, safe, progress, W, C)
    for j in range(30):
        a, b = int(seg_off[j]), int(seg_off[j + 1])
        p = int(progress[j])
        total = int(dur[a + p:b].sum())
        peak = int(mem[a + p:b].max())
        want = np.where((total <= W) & (peak <= C), b - a, -1)
        np.testing.assert_array_equal(cut[:, j], want)


def test_finished_and_empty_jobs_never_fit(oracle):
    seg_off = np.array([0, 0, 3, 3, 5], dtype=np.int64)      # jobs 0 and 2 are empty
    dur = np.array([1, 1, 1, 2, 2], dtype=np.int32)
    mem = np.array([1, 1, 1, 1, 1], dtype=np.int32)
    safe = np.ones(5, dtype=np.uint8)
    progress = np.array([0, 3, 0, 0], dtype=np.int32)        # job 1 is finished
    W = np.array([INT_MAX, 0, 3], dtype=np.int32)
    C = np.array([INT_MAX, 5, 5], dtype=np.int32)
    cut, bits = oracle.fit(seg_off, dur, mem, safe, progress, W, C)
    np.testing.assert_array_equal(cut[:, :3], -1)
    np.testing.assert_array_equal(cut[:, 3], [2, -1, 1])
    np.testing.assert_array_equal(bits[:, 0], [8, 0, 8])


def test_illustrative_scenario_from_the_paper(oracle):
    """Sec. 3.9 'Illustrative Scenario': a 40 GB training job cannot get a whole device,
    a ten-minute gap on a 20 GB slice is advertised, and the job answers with a subjob
    that fits the slice and the window and ends on a checkpoint.  The same job without
    internal subjob boundaries (a monolith) must decline.  The profile is a stand-in of
    our own (the paper gives the situation, not numbers beyond 40 GB / 20 GB / 10 min)."""
    with open(os.path.join(GOLDEN, "illustrative_scenario.json")) as f:
        sc = json.load(f)
    dur = np.array(sc["dur_s"], dtype=np.int32)
    mem = np.array(sc["mem_mib"], dtype=np.int32)
    safe = np.array(sc["safe"], dtype=np.uint8)
    seg_off = np.array([0, len(dur)], dtype=np.int64)
    progress = np.array([0], dtype=np.int32)
    W = np.array([sc["gap_window_s"]], dtype=np.int32)
    C = np.array([sc["gap_capacity_mib"]], dtype=np.int32)
    assert mem.max() == 40960 and C[0] == 20480 and W[0] == 600
    cut, _ = oracle.fit(seg_off, dur, mem, safe, progress, W, C)
    assert cut[0, 0] == sc["expected_cut"]
    c = int(cut[0, 0])
    assert dur[:c].sum() <= 600 and mem[:c].max() <= 20480 and safe[c - 1] == 1
    mono = np.zeros_like(safe)
    cut_m, _ = oracle.fit(seg_off, dur, mem, mono, progress, W, C)
    assert cut_m[0, 0] == -1


@pytest.mark.parametrize("name", ["large", "stress"])
def test_fullsize_digest_files_come_from_this_oracle(oracle, name):
    """The stored full-size digests (tests/golden/make_fullsize_digest.py) are what the oracle
    gives today: two of their blocks recomputed here."""
    import importlib.util
    path = os.path.join(GOLDEN, f"fullsize_digest_{name}.json")
    with open(path) as f:
        gold = json.load(f)
    spec = importlib.util.spec_from_file_location("make_fullsize_digest",
                                                  os.path.join(GOLDEN, "make_fullsize_digest.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    wl = make_workload(name, gold["seed"])
    assert len(gold["blocks"]) == (wl.n_gaps + gold["block"] - 1) // gold["block"]
    par = oracle.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override, 0)
    pd, pp, _ = oracle.prepare(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress)
    for b in (0, len(gold["blocks"]) - 1):
        g0 = b * gold["block"]
        W = np.ascontiguousarray(wl.W[g0:g0 + gold["block"]])
        C = np.ascontiguousarray(wl.C[g0:g0 + gold["block"]])
        cut, _ = oracle.fit(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, W, C, False)
        cj, cc, cs = oracle.select(cut, wl.seg_off, pd, pp, par, wl.wait, wl.sla_class)
        assert mod.block_digest(cut, g0, cj, cc, cs) == gold["blocks"][b]
