"""TEST INFRASTRUCTURE: from-scratch brute force in pure Python, tiny inputs only.

An independent restatement of the definitions used to pin oracle/sja_oracle.c:
nothing is accumulated incrementally, nothing is assumed monotone, every
candidate boundary is tested on its own, the arg-max is a full sort and the
conflict rounds are simulated with explicit sets.  Python integers are
unbounded, so no overflow question arises here.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

EFFICIENCY, FAIRNESS, SLA, MIXED = 0, 1, 2, 3


def job_slices(seg_off, arr, j):
    return [int(x) for x in arr[int(seg_off[j]):int(seg_off[j + 1])]]


def fit_one(dur: Sequence[int], mem: Sequence[int], safe: Sequence[int], p: int,
            W: int, C: int) -> int:
    """Largest safe boundary b in (p, L] whose subjob [p, b) fits (Sec. 3.8-3.9)."""
    L = len(dur)
    for b in range(L, p, -1):                     # every boundary, longest first
        is_safe = (b == L) or bool(safe[b - 1])
        if not is_safe:
            continue
        total = sum(dur[p:b])                     # recomputed from scratch
        peak = max(mem[p:b])
        if total <= W and peak <= C:
            return b
    return -1


def fit_all(seg_off, dur, mem, safe, progress, W, C) -> List[List[int]]:
    J = len(seg_off) - 1
    out = []
    for g in range(len(W)):
        row = []
        for j in range(J):
            row.append(fit_one(job_slices(seg_off, dur, j), job_slices(seg_off, mem, j),
                               job_slices(seg_off, safe, j), int(progress[j]),
                               int(W[g]), int(C[g])))
        out.append(row)
    return out


def key_of(policy: int, sub_dur: int, sub_peak: int, wait: int, cls: int, wait_scale: int,
           sla_weight: Sequence[int], class0_override: int, F: Optional[int] = None) -> Tuple[int, int, int]:
    """F defaults to the rectangle duration x peak; the area variant passes its own F."""
    if F is None:
        F = sub_dur * sub_peak
    if policy == EFFICIENCY:
        return (0, F, 0)
    if policy == FAIRNESS:
        return (0, F * (wait_scale + wait), 0)
    if policy == SLA:
        return (1 if (class0_override and cls == 0) else 0, F * sla_weight[cls], 0)
    if policy == MIXED:
        return (2 - cls, F * (wait_scale + wait), F)
    raise ValueError(policy)


def select_gap(cut_row, seg_off, dur, mem, progress, wait, sla_class, policy,
               wait_scale=1000, sla_weight=(4, 2, 1), class0_override=1,
               held: Optional[set] = None, by_area: bool = False):
    """(job, cut, score) for one gap: sort every candidate, take the first.
    by_area: F = sum of dur * mem over the subjob instead of its duration x peak."""
    cands = []
    for j, c in enumerate(cut_row):
        if c < 0 or (held is not None and j in held):
            continue
        d = job_slices(seg_off, dur, j)
        m = job_slices(seg_off, mem, j)
        p = int(progress[j])
        F = sum(x * y for x, y in zip(d[p:c], m[p:c])) if by_area else None
        key = key_of(policy, sum(d[p:c]), max(m[p:c]), int(wait[j]), int(sla_class[j]),
                     wait_scale, sla_weight, class0_override, F)
        cands.append((key, j, c))
    if not cands:
        return (-1, -1, 0)
    cands.sort(key=lambda t: (-t[0][0], -t[0][1], -t[0][2], t[1]))
    key, j, c = cands[0]
    return (j, c, key[1])


def resolve(cut, seg_off, dur, mem, progress, wait, sla_class, policy, max_rounds=0,
            wait_scale=1000, sla_weight=(4, 2, 1), class0_override=1, by_area: bool = False):
    """Literal simulation of the grant rounds with explicit sets."""
    G = len(cut)
    J = len(seg_off) - 1
    grant = {g: None for g in range(G)}
    held = set()
    holder = {}
    cap = max_rounds if max_rounds > 0 else min(G, J) + 1
    rounds, stable = 0, 0
    for _ in range(cap):
        choice = {}
        for g in range(G):
            if grant[g] is not None:
                continue
            j, c, s = select_gap(cut[g], seg_off, dur, mem, progress, wait, sla_class, policy,
                                 wait_scale, sla_weight, class0_override, held, by_area)
            if j >= 0:
                choice[g] = (j, c, s)
        rounds += 1
        if not choice:
            stable = 1
            break
        wanted = {}
        for g, (j, c, s) in choice.items():
            wanted.setdefault(j, []).append(g)
        lost = 0
        for j, gaps in wanted.items():
            g_star = min(gaps)
            grant[g_star] = choice[g_star]
            held.add(j)
            holder[j] = g_star
            lost += len(gaps) - 1
        if lost == 0:
            stable = 1
            break
    grant_job = [grant[g][0] if grant[g] else -1 for g in range(G)]
    grant_cut = [grant[g][1] if grant[g] else -1 for g in range(G)]
    grant_score = [grant[g][2] if grant[g] else 0 for g in range(G)]
    job_gap = [holder.get(j, -1) for j in range(J)]
    return grant_job, grant_cut, grant_score, job_gap, rounds, stable


def advance(seg_off, dur, mem, W, C, grant_job, grant_cut, progress, wait, wait_step):
    """One tick's bookkeeping straight from the raw segments (Sec. 3.1, 3.5; metrics of Sec. 5):
    returns (progress', wait', [filled, offered, grants, finished])."""
    J = len(seg_off) - 1
    prog = [int(x) for x in progress]
    wt = [int(x) for x in wait]
    took = {}
    for g, j in enumerate(grant_job):
        if int(j) >= 0:
            assert int(j) not in took
            took[int(j)] = g
    filled = 0
    for j, g in took.items():
        d = job_slices(seg_off, dur, j)[prog[j]:int(grant_cut[g])]
        m = job_slices(seg_off, mem, j)[prog[j]:int(grant_cut[g])]
        filled += sum(d) * max(m)
    offered = sum(max(int(w), 0) * max(int(c), 0) for w, c in zip(W, C))
    finished = 0
    for j in range(J):
        L = int(seg_off[j + 1]) - int(seg_off[j])
        if j in took:
            prog[j] = int(grant_cut[took[j]])
            wt[j] = 0
        elif prog[j] < L:
            wt[j] = min(wt[j] + wait_step, 2**31 - 1)
        finished += prog[j] >= L
    return prog, wt, [filled, offered, len(took), finished]


def fit_one_limited(dur, mem, safe, p, W, C, tau_min=0, tau_max=None, power=None, power_cap=None,
                    deadline=None, now=0) -> int:
    """fit_one under the admission limits of Sec. 4.3 (duration bounds) and Sec. 4.4 (power cap,
    deadline): every test written out for every boundary, longest first."""
    L = len(dur)
    for b in range(L, p, -1):
        if not ((b == L) or bool(safe[b - 1])):
            continue
        total = sum(dur[p:b])
        ok = total <= W and max(mem[p:b]) <= C
        if tau_max is not None:
            ok = ok and total <= tau_max
        if b != L:
            ok = ok and total >= tau_min
        if power is not None:
            ok = ok and max(power[p:b]) <= power_cap
        if deadline is not None:
            ok = ok and now + total <= deadline
        if ok:
            return b
    return -1


def cover_one(peak: int, cap_set: Sequence[int]):
    """Smallest capacity of the set that covers the peak (Sec. 3.9), or None."""
    fits = [int(c) for c in cap_set if int(c) >= peak]
    return min(fits) if fits else None


def fit_one_hysteresis(dur, mem, safe, p, W, C, cap_set, min_gain, tau_min=0, tau_max=None, power=None,
                       power_cap=None, deadline=None, now=0) -> int:
    """The hysteresis rule of Sec. 3.9 (safeguard ii) as a set definition: among the boundaries the
    pair admits, the longest one b* stands unless a shorter one maps to a covering capacity at least
    min_gain below that of b*; then the longest such shorter boundary is the cut."""
    L = len(dur)
    admitted = []
    for b in range(p + 1, L + 1):
        if not ((b == L) or bool(safe[b - 1])):
            continue
        total = sum(dur[p:b])
        ok = total <= W and max(mem[p:b]) <= C
        if tau_max is not None:
            ok = ok and total <= tau_max
        if b != L:
            ok = ok and total >= tau_min
        if power is not None:
            ok = ok and max(power[p:b]) <= power_cap
        if deadline is not None:
            ok = ok and now + total <= deadline
        if ok:
            admitted.append(b)
    if not admitted:
        return -1
    b_star = max(admitted)
    if not len(cap_set):
        return b_star
    inf = float("inf")
    cov = {}
    for b in admitted:
        c = cover_one(max(mem[p:b]), cap_set)
        cov[b] = inf if c is None else c
    worth = [b for b in admitted if b < b_star and cov[b] != inf
             and (cov[b_star] == inf or cov[b_star] - cov[b] >= min_gain)]
    return max(worth) if worth else b_star
