"""Small random-profile builders shared by the CPU tests (inputs only)."""
import numpy as np


def random_jobs(rng, n_jobs, l_lo, l_hi, *, d_hi=9, m_hi=9, safe_p=0.4, allow_done=True):
    lens = rng.integers(l_lo, l_hi + 1, size=n_jobs)
    seg_off = np.zeros(n_jobs + 1, dtype=np.int64)
    np.cumsum(lens, out=seg_off[1:])
    S = int(seg_off[-1])
    dur = rng.integers(1, d_hi + 1, size=S).astype(np.int32)
    mem = rng.integers(0, m_hi + 1, size=S).astype(np.int32)
    safe = (rng.random(S) < safe_p).astype(np.uint8)
    hi = lens + 1 if allow_done else np.maximum(lens, 1)
    progress = (rng.random(n_jobs) * hi).astype(np.int32)
    progress = np.minimum(progress, lens).astype(np.int32)
    return seg_off, dur, mem, safe, progress


def random_gaps(rng, n_gaps, w_hi, c_hi):
    W = rng.integers(0, w_hi + 1, size=n_gaps).astype(np.int32)
    C = rng.integers(0, c_hi + 1, size=n_gaps).astype(np.int32)
    return W, C


def random_prefs(rng, n_jobs, wait_hi=5):
    wait = rng.integers(0, wait_hi + 1, size=n_jobs).astype(np.int32)
    cls = rng.integers(0, 3, size=n_jobs).astype(np.uint8)
    return wait, cls
