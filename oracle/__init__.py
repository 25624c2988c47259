"""CPU oracle for the constrained layer-wise compression dynamic program (Sec. 3.2, App. A).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the benchmark's
CPU-baseline leg.  It shares nothing with the GPU library and never imports it.

``spdy_dp_ref.c``  -- Alg. 1 in plain single-threaded C (fp32, strict "<", smallest level wins).
``brute_force.c``  -- exhaustive enumeration of Eq. 1 for tiny instances (the definition).
This module compiles both with gcc into ``liboracle.so`` next to the sources and exposes them
through ctypes on NumPy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SOURCES = [os.path.join(_HERE, "spdy_dp_ref.c"), os.path.join(_HERE, "brute_force.c")]
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_lib = None

# no -ffast-math, no contraction: every add is one IEEE fp32 add; SSE keeps subnormals
_CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-fno-fast-math", "-ffp-contract=off",
           "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (only if the library is missing or older than a source)."""
    stale = force or not os.path.exists(_LIB_PATH) or any(
        os.path.getmtime(s) > os.path.getmtime(_LIB_PATH) for s in _SOURCES)
    if stale:
        tmp = _LIB_PATH + f".tmp{os.getpid()}"
        subprocess.run(["gcc", *_CFLAGS, *_SOURCES, "-o", tmp, "-lm"], check=True)
        os.replace(tmp, _LIB_PATH)
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i32p = ctypes.POINTER(ctypes.c_int32)
        f32p = ctypes.POINTER(ctypes.c_float)
        i16p = ctypes.POINTER(ctypes.c_int16)
        i64p = ctypes.POINTER(ctypes.c_int64)
        lib.spdy_dp_solve_ref.restype = ctypes.c_int
        lib.spdy_dp_solve_ref.argtypes = [i32p, f32p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                          ctypes.c_int, i16p, f32p]
        lib.spdy_dp_solve_sens_ref.restype = ctypes.c_int
        lib.spdy_dp_solve_sens_ref.argtypes = [i32p, f32p, f32p, ctypes.c_int, ctypes.c_int,
                                               ctypes.c_int, ctypes.c_int, i16p, f32p]
        lib.spdy_dp_tables_ref.restype = ctypes.c_int
        lib.spdy_dp_tables_ref.argtypes = [i32p, f32p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                           f32p, i32p, i16p, f32p]
        lib.spdy_brute_force.restype = ctypes.c_int
        lib.spdy_brute_force.argtypes = [i32p, f32p, ctypes.c_int, ctypes.c_int, ctypes.c_int64,
                                         i16p, f32p, i64p, i64p]
        _lib = lib
    return _lib


def _ptr(a: np.ndarray, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _check(tau, err):
    tau = np.ascontiguousarray(tau, dtype=np.int32)
    err = np.ascontiguousarray(err, dtype=np.float32)
    if tau.ndim != 2:
        raise ValueError("tau must be [L, S]")
    if err.ndim == 2:
        err = err[None]
    if err.ndim != 3 or err.shape[1:] != tau.shape:
        raise ValueError("err must be [K, L, S] matching tau [L, S]")
    return tau, err


def solve_ref_status(tau, err, B: int):
    """Raw call: returns (status, profile int16[K,L], cost fp32[K]) without raising."""
    tau, err = _check(tau, err)
    K, L, S = err.shape
    profile = np.full((K, L), -2, dtype=np.int16)
    cost = np.full((K,), np.nan, dtype=np.float32)
    st = _load().spdy_dp_solve_ref(_ptr(tau, ctypes.c_int32), _ptr(err, ctypes.c_float), K, L, S,
                                   int(B), _ptr(profile, ctypes.c_int16),
                                   _ptr(cost, ctypes.c_float))
    return st, profile, cost


def solve_ref(tau, err, B: int, threads: int = 1):
    """Alg. 1 for K candidates.  Returns ``(profile int16[K,L], cost fp32[K])``.

    ``threads > 1`` runs the same single-threaded routine on disjoint candidate ranges from a
    thread pool (ctypes releases the GIL); the arithmetic per candidate is unchanged.
    """
    tau, err = _check(tau, err)
    K = err.shape[0]
    threads = max(1, min(int(threads), K))
    if threads == 1:
        st, profile, cost = solve_ref_status(tau, err, B)
        if st != 0:
            raise ValueError(f"spdy_dp_solve_ref failed with status {st}")
        return profile, cost
    bounds = np.linspace(0, K, threads + 1).astype(int)
    with ThreadPoolExecutor(threads) as pool:
        parts = list(pool.map(lambda i: solve_ref_status(tau, err[bounds[i]:bounds[i + 1]], B),
                              range(threads)))
    for st, _, _ in parts:
        if st != 0:
            raise ValueError(f"spdy_dp_solve_ref failed with status {st}")
    return (np.concatenate([p for _, p, _ in parts]), np.concatenate([c for _, _, c in parts]))


def solve_sens_ref(tau, c, w, B: int):
    """Alg. 1 on err[k,l,s] = fl32(c[k,l] * w[s]) (Eq. 4).  Returns ``(profile, cost)``."""
    tau = np.ascontiguousarray(tau, dtype=np.int32)
    c = np.ascontiguousarray(c, dtype=np.float32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    if tau.ndim != 2 or c.ndim != 2 or w.ndim != 1 or c.shape[1] != tau.shape[0] \
            or w.shape[0] != tau.shape[1]:
        raise ValueError("tau [L, S], c [K, L], w [S] expected")
    K, L = c.shape
    S = w.shape[0]
    profile = np.full((K, L), -2, dtype=np.int16)
    cost = np.full((K,), np.nan, dtype=np.float32)
    st = _load().spdy_dp_solve_sens_ref(_ptr(tau, ctypes.c_int32), _ptr(c, ctypes.c_float),
                                        _ptr(w, ctypes.c_float), K, L, S, int(B),
                                        _ptr(profile, ctypes.c_int16), _ptr(cost, ctypes.c_float))
    if st != 0:
        raise ValueError(f"spdy_dp_solve_sens_ref failed with status {st}")
    return profile, cost


def solve_budgets_ref(tau, err, budgets, threads: int = 1):
    """Alg. 1 solved separately for every budget: ``(profile int16[J,K,L], cost fp32[J,K])``."""
    out = [solve_ref(tau, err, int(b), threads=threads) for b in budgets]
    return np.stack([p for p, _ in out]), np.stack([c for _, c in out])


def tables_ref(tau, err, B: int):
    """Alg. 1 for one candidate, returning ``(D fp32[L,B+1], P int32[L,B+1], profile, cost)``."""
    tau, err = _check(tau, err)
    if err.shape[0] != 1:
        raise ValueError("tables_ref takes one candidate")
    _, L, S = err.shape
    D = np.empty((L, B + 1), dtype=np.float32)
    P = np.empty((L, B + 1), dtype=np.int32)
    profile = np.empty((L,), dtype=np.int16)
    cost = np.empty((1,), dtype=np.float32)
    st = _load().spdy_dp_tables_ref(_ptr(tau, ctypes.c_int32), _ptr(err, ctypes.c_float), L, S,
                                    int(B), _ptr(D, ctypes.c_float), _ptr(P, ctypes.c_int32),
                                    _ptr(profile, ctypes.c_int16), _ptr(cost, ctypes.c_float))
    if st != 0:
        raise ValueError(f"spdy_dp_tables_ref failed with status {st}")
    return D, P, profile, cost[0]


def brute_force(tau, err, B: int):
    """Enumerate all S^L profiles of ONE candidate (Eq. 1).

    Returns ``(profile int16[L], cost fp32, time int, n_best int)``; infeasible: (-1.., inf, -1, 0).
    """
    tau, err = _check(tau, err)
    if err.shape[0] != 1:
        raise ValueError("brute_force takes one candidate")
    _, L, S = err.shape
    profile = np.empty((L,), dtype=np.int16)
    cost = ctypes.c_float()
    time = ctypes.c_int64()
    n = ctypes.c_int64()
    st = _load().spdy_brute_force(_ptr(tau, ctypes.c_int32), _ptr(err, ctypes.c_float), L, S,
                                  int(B), _ptr(profile, ctypes.c_int16), ctypes.byref(cost),
                                  ctypes.byref(time), ctypes.byref(n))
    if st != 0:
        raise ValueError("brute force refused the instance (too large or bad arguments)")
    return profile, np.float32(cost.value), int(time.value), int(n.value)
