"""The oracle under the compiler's sanitizers: oracle/sja_oracle.c is built with
-fsanitize=address,undefined into an executable of its own (oracle/sanitize_driver.c) and run on
tiny random cases whose answers come from the from-scratch Python brute force, on buffers of
exactly the documented sizes.  Any out-of-bounds access, signed overflow or misaligned access in
the oracle ends the run with a report; any value that differs from the brute force fails it."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import brute
from helpers import random_gaps, random_jobs, random_prefs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _case(rng, policy):
    n_jobs = int(rng.integers(1, 7))
    n_gaps = int(rng.integers(1, 6))
    seg_off, dur, mem, safe, progress = random_jobs(rng, n_jobs, 0, 7)
    W, C = random_gaps(rng, n_gaps, 30, 9)
    wait, cls = random_prefs(rng, n_jobs)
    max_rounds = int(rng.integers(0, 3))
    cut = brute.fit_all(seg_off, dur, mem, safe, progress, W, C)
    cand = [brute.select_gap(cut[g], seg_off, dur, mem, progress, wait, cls, policy, 2, (4, 2, 1), 1)
            for g in range(n_gaps)]
    gj, gc, gs, jg, rounds, stable = brute.resolve(cut, seg_off, dur, mem, progress, wait, cls, policy,
                                                   max_rounds, 2, (4, 2, 1), 1)
    head = [n_jobs, n_gaps, len(dur), policy, 2, 4, 2, 1, 1, max_rounds]
    parts = [head, seg_off, dur, mem, safe, progress, W, C, wait, cls,
             [c for row in cut for c in row], [c[0] for c in cand], [c[1] for c in cand], [c[2] for c in cand],
             gj, gc, gs, jg, [rounds, stable]]
    return " ".join(str(int(x)) for part in parts for x in part)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_is_clean_under_address_and_undefined_sanitizers(tmp_path):
    exe = tmp_path / "oracle_sanitized"
    cmd = ["gcc", "-O1", "-g", "-std=c99", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", "-static-libasan", "-Wall", "-Wextra", "-o", str(exe),
           os.path.join(ROOT, "oracle", "sja_oracle.c"), os.path.join(ROOT, "oracle", "sanitize_driver.c")]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    rng = np.random.default_rng(20250919)
    cases = [_case(rng, policy) for policy in (0, 1, 2, 3) for _ in range(150)]
    path = tmp_path / "cases.txt"
    path.write_text(f"{len(cases)}\n" + "\n".join(cases) + "\n")
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([str(exe), str(path)], capture_output=True, text=True, env=env)
    assert run.returncode == 0, run.stdout + run.stderr
    assert f"{len(cases)} cases equal" in run.stdout
