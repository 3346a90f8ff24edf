"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

oracle/sanitize_harness.c includes galv_oracle.c, is built here with
-fsanitize=address,undefined -fno-sanitize-recover=all and fed seeded instances — among
them the edge cases the GPU parity tests rely on (budget 0, memory INT32_MAX, one layer,
one strategy, no selector array, costs near the 2^62 precondition).  A memory error or
undefined behaviour inside the oracle aborts the run; its output must equal what the
ordinary -O2 build returns for the same instances."""
import os
import shutil
import subprocess

import numpy as np
import pytest

import oracle
from paper_2211_13878_amd import workloads

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "sanitize_harness.c")


@pytest.fixture(scope="module")
def harness(tmp_path_factory):
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    exe = str(tmp_path_factory.mktemp("san") / "galv_oracle_san")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c99", "-Wall", "-Wextra",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-o", exe, SRC])
    assert b"__asan_init" in subprocess.check_output(["nm", "-D", exe]) + subprocess.check_output(["nm", exe])
    return exe


def cases():
    rng = np.random.default_rng(2024)
    out = []
    for i in range(40):
        L, S = int(rng.integers(1, 7)), int(rng.integers(1, 9))
        E = int(rng.integers(0, 60))
        w = workloads.random_workload(int(rng.integers(1 << 30)), 1, L, S, E, nR=int(rng.integers(1, 4)),
                                      m_range=(0, 12), c_range=(0, 30), r_range=(0, 9),
                                      infeasible=0.1, zero_diagonal=bool(i % 2))
        c, m, R, r_idx, budget = w.instance(0)
        if i % 7 == 0:
            m = m.copy(); m.flat[0] = 2**31 - 1            # e - m must not wrap
        if i % 5 == 0:
            budget = 0
        if i % 11 == 0:
            c = c.astype(np.int64) * ((1 << 58) // 31 // max(1, L))   # sums just below 2^62
        out.append((c, m, R, None if i % 3 == 0 else r_idx, budget, i % 2))
    return out


def test_sanitized_oracle_agrees_with_the_ordinary_build(harness):
    lines, expect = [], []
    for c, m, R, r_idx, budget, tables in cases():
        L, S = c.shape
        nR = R.shape[0]
        nums = [L, S, nR, budget, int(r_idx is not None), tables] + c.ravel().tolist() + m.ravel().tolist() + \
            R.ravel().tolist() + ([] if r_idx is None else r_idx.tolist())
        lines.append(" ".join(str(int(x)) for x in nums))
        ref = oracle.solve(c, m, R, r_idx, budget, want_C_last=bool(tables), want_bp=bool(tables))
        sums = (int((ref.C_last % (1 << 31)).sum()), int((ref.bp.astype(np.int64) + 1).sum())) if tables else (0, 0)
        expect.append([0, ref.best_cost, ref.best_last, ref.n_tied] + [int(s) for s in ref.plan] + list(sums))
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([harness], input="\n".join(lines) + "\n", capture_output=True, text=True, env=env)
    assert run.returncode == 0, run.stderr[-2000:]
    got = [[int(x) for x in ln.split()] for ln in run.stdout.strip().split("\n")]
    assert got == expect
    assert any(e[1] == oracle.INF for e in expect) and any(e[1] < oracle.INF for e in expect)


def test_bad_arguments_are_refused_not_dereferenced(harness):
    # r_idx out of range: the oracle must return -1 before using it as an index
    line = "2 2 1 3 1 0  1 1 1 1  0 0 0 0  0 0 0 0  0 5"
    run = subprocess.run([harness], input=line + "\n", capture_output=True, text=True,
                         env=dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0"))
    assert run.returncode == 0, run.stderr[-2000:]
    assert run.stdout.split()[0] == "-1"
