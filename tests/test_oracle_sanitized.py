"""The oracle's C routines under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

The two oracle sources are compiled once more, with ``-fsanitize=address,undefined`` and a small
driver (``oracle_sanitized_main.c``), into an executable that solves a batch of instances (random
shapes, the edge cases of the problem, the hand-worked fixtures).  The run must end cleanly (an
out-of-bounds access, a leak or undefined arithmetic aborts it) and must print exactly what the
ordinary build returns.
"""
import os
import shutil
import subprocess

import numpy as np
import pytest

import oracle
import workloads

HERE = os.path.dirname(os.path.abspath(__file__))
ORACLE = os.path.join(os.path.dirname(HERE), "oracle")
CFLAGS = ["-O1", "-g", "-std=c11", "-fno-omit-frame-pointer", "-fno-fast-math",
          "-ffp-contract=off", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
          "-static-libasan", "-Wall", "-Wextra"]


@pytest.fixture(scope="module")
def sanitized(tmp_path_factory):
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    exe = str(tmp_path_factory.mktemp("san") / "oracle_sanitized")
    subprocess.run(["gcc", *CFLAGS, os.path.join(HERE, "oracle_sanitized_main.c"),
                    os.path.join(ORACLE, "spdy_dp_ref.c"), os.path.join(ORACLE, "brute_force.c"),
                    "-o", exe, "-lm"], check=True)
    return exe


def instances():
    rng = np.random.default_rng(4711)
    out = []
    for case in range(60):
        K = int(rng.integers(1, 4))
        L = int(rng.integers(1, 6))
        S = int(rng.integers(1, 6))
        B = int(rng.choice([0, 1, 2, 7, 30, 64, 200]))
        kw = dict(tau_max=max(1, B // 2 + 1), zero_tau_frac=float(rng.choice([0, 0.3])),
                  over_budget_frac=float(rng.choice([0, 0.3])),
                  inf_err_frac=float(rng.choice([0, 0.2])),
                  integer_err=int(rng.choice([0, 3])) or None,
                  huge_tau_frac=0.1 if case % 7 == 0 else 0.0)
        tau, err, _ = workloads.random_instance(rng, K, L, S, B, **kw)
        out.append((tau, err, B, S ** L <= 4000))
    # no feasible profile at all; a single cell; one long row
    out.append((np.array([[5, 6], [7, 9]], dtype=np.int32),
                np.zeros((2, 2, 2), dtype=np.float32), 3, True))
    out.append((np.zeros((1, 1), dtype=np.int32), np.ones((1, 1, 1), dtype=np.float32), 0, True))
    tau, err, B = workloads.generate(workloads.CONFIGS["tiny"], K=2)
    out.append((tau, err, B, False))
    return out


def encode(batch):
    lines = []
    for tau, err, B, brute in batch:
        K, L, S = err.shape
        lines.append(f"{K} {L} {S} {B} {int(brute)}")
        lines.append(" ".join(str(int(x)) for x in tau.ravel()))
        lines.append(" ".join(f"{x:08x}" for x in err.ravel().view(np.uint32)))
    return "\n".join(lines) + "\n"


def expected(batch):
    lines = []
    for tau, err, B, brute in batch:
        K, L, S = err.shape
        st, p, c = oracle.solve_ref_status(tau, err, B)
        lines.append(f"status {st}")
        if st == 0:
            for k in range(K):
                lines.append(" ".join([f"{c[k:k + 1].view(np.uint32)[0]:08x}"] +
                                      [str(int(s)) for s in p[k]]))
            D, P, _, _ = oracle.tables_ref(tau, err[0], B)
            for l in range(L):
                lines.append("D " + " ".join(f"{x:08x}" for x in D[l].view(np.uint32)))
                lines.append("P " + " ".join(str(int(x)) for x in P[l]))
            cs, w = err[:, :, 0], err[0, 0, :]
            if np.isfinite(cs).all() and np.isfinite(w).all():
                _, c2 = oracle.solve_sens_ref(tau, np.ascontiguousarray(cs),
                                              np.ascontiguousarray(w), B)
                lines.append("sens 0 " + " ".join(f"{x:08x}" for x in c2.view(np.uint32)))
        if brute:
            bp, bc, bt, nb = oracle.brute_force(tau, err[:1], B)
            lines.append(" ".join([f"brute 0 {np.array([bc]).view(np.uint32)[0]:08x} {bt} {nb}"] +
                                  [str(int(s)) for s in bp]))
    return lines


def test_oracle_runs_clean_under_sanitizers(sanitized):
    batch = instances()
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([sanitized], input=encode(batch), capture_output=True, text=True, env=env,
                         timeout=300)
    assert res.returncode == 0, res.stderr[-4000:]
    assert "ERROR" not in res.stderr and "runtime error" not in res.stderr, res.stderr[-4000:]
    got = res.stdout.strip().split("\n")
    want = expected(batch)
    assert len(got) == len(want)
    for i, (g, w) in enumerate(zip(got, want)):
        assert g.split() == w.split(), f"line {i}: {g[:200]} != {w[:200]}"


def test_sanitizers_are_armed(sanitized, tmp_path):
    """The same flags do catch a planted out-of-bounds write (a tiny C program compiled here, on
    the CPU), so a clean run above means something."""
    src = tmp_path / "oob.c"
    src.write_text("#include <stdlib.h>\nint main(void){volatile int *p = malloc(8 * sizeof(int));"
                   " p[8] = 1; free((void *)p); return 0;}\n")
    exe = str(tmp_path / "oob")
    subprocess.run(["gcc", *CFLAGS, str(src), "-o", exe], check=True)
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=60)
    assert res.returncode != 0
    assert "heap-buffer-overflow" in res.stderr or "runtime error" in res.stderr
