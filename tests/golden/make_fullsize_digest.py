"""Writes tests/golden/fullsize_digest_<config>.json: digests of the ORACLE's fit and select
outputs for every gap of a full-size config, one record per block of 256 gaps (in the caller's
gap order).  Calls only gen/ and oracle/.  The GPU tests recompute the same digests from the
library's outputs, which compares whole outputs at sizes where the oracle takes minutes.

    python tests/golden/make_fullsize_digest.py large stress
    python tests/golden/make_fullsize_digest.py --resolve large stress   (adds the grants; keeps the whole
                                                                         cut matrix in host memory, hours at Stress)
    python tests/golden/make_fullsize_digest.py --resolve --caps=8 stress   (only these round caps; entries for
                                                                         other caps already in the file are kept)

Per block b (gaps g = 256 b .. 256 b + 255, jobs j), all sums in wrapping int64:
    interested   number of pairs with cut >= 0
    cut_sum      sum of cut
    cut_mix      sum of (cut + 2) * (j + 1) * (g + 1)       (catches moved rows and columns)
    cand_job     sum of cand_job * (g + 1)
    cand_cut     sum of cand_cut * (g + 1)
    cand_score   sum of cand_score
With --resolve, "resolve" holds, for the round cap of the config, for 8 and for 0 (until stable): rounds, stable,
the number of grants and sum grant_job * (g + 1), sum grant_cut * (g + 1), sum grant_score,
sum job_gap * (j + 1), all in wrapping int64.
"""
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

BLOCK = 256


def block_digest(cut, g0, cand_job, cand_cut, cand_score):
    rows, J = cut.shape
    c = cut.astype(np.int64)
    jw = np.arange(1, J + 1, dtype=np.int64)[None, :]
    gw = np.arange(g0 + 1, g0 + rows + 1, dtype=np.int64)
    with np.errstate(over="ignore"):
        mix = ((c + 2) * jw * gw[:, None]).sum(dtype=np.int64)
        return {"interested": int((cut >= 0).sum()), "cut_sum": int(c.sum(dtype=np.int64)), "cut_mix": int(mix),
                "cand_job": int((cand_job.astype(np.int64) * gw).sum(dtype=np.int64)),
                "cand_cut": int((cand_cut.astype(np.int64) * gw).sum(dtype=np.int64)),
                "cand_score": int(cand_score.sum(dtype=np.int64))}


def grant_digest(gj, gc, gs, jg, rounds, stable):
    gw = np.arange(1, len(gj) + 1, dtype=np.int64)
    jw = np.arange(1, len(jg) + 1, dtype=np.int64)
    with np.errstate(over="ignore"):
        return {"rounds": int(rounds), "stable": int(stable), "grants": int((gj >= 0).sum()),
                "grant_job": int((gj.astype(np.int64) * gw).sum(dtype=np.int64)),
                "grant_cut": int((gc.astype(np.int64) * gw).sum(dtype=np.int64)),
                "grant_score": int(gs.sum(dtype=np.int64)),
                "job_gap": int((jg.astype(np.int64) * jw).sum(dtype=np.int64))}


def main(names):
    import oracle as O
    from gen import make_workload
    with_resolve = "--resolve" in names
    caps_arg = [n.split("=", 1)[1] for n in names if n.startswith("--caps=")]
    names = [n for n in names if not n.startswith("--")] or ["large", "stress"]
    for name in names:
        wl = make_workload(name, 0)
        par = O.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override, 0)
        pd, pp, _ = O.prepare(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress)
        blocks = []
        whole = np.empty((wl.n_gaps, wl.n_jobs), dtype=np.int32) if with_resolve else None
        t0 = time.time()
        for g0 in range(0, wl.n_gaps, BLOCK):
            W = np.ascontiguousarray(wl.W[g0:g0 + BLOCK])
            C = np.ascontiguousarray(wl.C[g0:g0 + BLOCK])
            cut, _ = O.fit(wl.seg_off, wl.dur, wl.mem, wl.safe, wl.progress, W, C, False)
            cj, cc, cs = O.select(cut, wl.seg_off, pd, pp, par, wl.wait, wl.sla_class)
            blocks.append(block_digest(cut, g0, cj, cc, cs))
            if whole is not None:
                whole[g0:g0 + BLOCK] = cut
            if (g0 // BLOCK) % 16 == 0:
                print(f"{name}: gap {g0} of {wl.n_gaps}, {time.time() - t0:.0f} s", flush=True)
        out = {"config": name, "seed": 0, "n_gaps": wl.n_gaps, "n_jobs": wl.n_jobs, "policy": int(wl.policy),
               "block": BLOCK, "source": "oracle/ (sjo_fit, sjo_select, sjo_resolve where present), written by tests/golden/make_fullsize_digest.py",
               "blocks": blocks}
        path = os.path.join(ROOT, "tests", "golden", f"fullsize_digest_{name}.json")
        if whole is not None:
            out["resolve"] = {}
            if os.path.exists(path):
                with open(path) as f:
                    old = json.load(f)
                if old.get("blocks") == blocks:
                    out["resolve"] = old.get("resolve", {})
            caps = {int(c) for c in caps_arg[0].split(",")} if caps_arg else {int(wl.max_rounds), 8, 0}
            for cap in sorted(caps, reverse=True):
                p2 = O.Params.make(wl.policy, wl.wait_scale, wl.sla_weight, wl.class0_override, cap)
                res = O.resolve(whole, wl.seg_off, pd, pp, p2, wl.wait, wl.sla_class)
                out["resolve"][str(cap)] = grant_digest(*res)
                print(f"{name}: resolve cap {cap}: {res[4]} rounds, {time.time() - t0:.0f} s", flush=True)
        with open(path, "w") as f:
            json.dump(out, f, indent=0)
        print("wrote", path, flush=True)


if __name__ == "__main__":
    main(sys.argv[1:])
