"""Pins for the CPU oracle (no GPU): the oracle is only trusted because these pass.

Each test ties the oracle to something other than itself: the plain definition of the problem
(Eq. 1) by exhaustive enumeration, a hand-worked instance, closed forms, textbook reductions,
an integer-programming routine, and invariants the problem statement implies.
"""
import itertools
import os
import time

import numpy as np
import pytest

import oracle
import workloads

F32 = np.float32


def fp32_sum_in_layer_order(err_k, profile):
    acc = None
    for l, s in enumerate(profile):
        e = F32(err_k[l, s])
        acc = e if acc is None else F32(acc + e)
    return acc


def profile_time(tau, profile):
    return int(sum(int(tau[l, s]) for l, s in enumerate(profile)))


def python_enumeration(tau, err_k, B):
    """Eq. 1 with itertools, fp32 sums in layer order; returns (cost, time, set of optimal
    profiles for that (cost, time))."""
    L, S = tau.shape
    best = None
    winners = []
    for prof in itertools.product(range(S), repeat=L):
        t = profile_time(tau, prof)
        if t > B:
            continue
        c = fp32_sum_in_layer_order(err_k, prof)
        if not np.isfinite(c):
            continue
        key = (c, t)
        if best is None or key < best:
            best, winners = key, [prof]
        elif key == best:
            winners.append(prof)
    if best is None:
        return F32(np.inf), -1, []
    return best[0], best[1], winners


# --------------------------------------------------------------------------- hand-worked fixture
def load_golden(path):
    tau, err, cases = [], [], []
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            tok = line.split()
            if tok[0] == "dims":
                L, S = int(tok[1]), int(tok[2])
            elif tok[0] == "tau":
                tau.append([int(x) for x in tok[1:]])
            elif tok[0] == "err":
                err.append([float(x) for x in tok[1:]])
            elif tok[0] == "case":
                cases.append((int(tok[1]), float(tok[2]), int(tok[3]), [int(x) for x in tok[4:]]))
    tau = np.array(tau, dtype=np.int32)
    err = np.array(err, dtype=np.float32)
    assert tau.shape == (L, S) and err.shape == (L, S)
    return tau, err, cases


def test_hand_worked_instance(golden_dir):
    tau, err, cases = load_golden(os.path.join(golden_dir, "hand_worked_L3_S3.txt"))
    assert len(cases) >= 10
    for B, cost, t, prof in cases:
        p, c = oracle.solve_ref(tau, err, B)
        assert c[0] == F32(cost), (B, c)
        assert p[0].tolist() == prof, (B, p)
        if t >= 0:
            assert profile_time(tau, p[0]) == t
        bp, bc, bt, nb = oracle.brute_force(tau, err, B)
        assert bc == F32(cost) and bt == t and bp.tolist() == prof
        assert nb == (1 if t >= 0 else 0)


# --------------------------------------------------------------------------- the enumerator itself
def test_enumerator_matches_itertools():
    rng = np.random.default_rng(11)
    for trial in range(40):
        L, S = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        B = int(rng.integers(0, 30))
        tau, err, _ = workloads.random_instance(
            rng, 1, L, S, B, tau_max=12, integer_err=4 if trial % 2 else None,
            zero_tau_frac=0.1, over_budget_frac=0.05, inf_err_frac=0.05)
        c, t, winners = python_enumeration(tau, err[0], B)
        bp, bc, bt, nb = oracle.brute_force(tau, err, B)
        assert bt == t and nb == len(winners)
        if t < 0:
            assert np.isinf(bc) and (bp == -1).all()
            continue
        assert bc.tobytes() == F32(c).tobytes()
        # key: smallest (s_L, ..., s_1)
        want = min(winners, key=lambda p: tuple(reversed(p)))
        assert tuple(bp.tolist()) == want


# --------------------------------------------------------------------------- Eq. 1 by enumeration
@pytest.mark.parametrize("seed", range(6))
def test_continuous_errors_against_enumeration(seed):
    """Random real errors: ties are (almost) absent.  Cost must be bit-equal to the least fp32
    layer-order sum; the profile must be optimal, and equal when the optimum is unique."""
    rng = np.random.default_rng(100 + seed)
    n_unique = 0
    for _ in range(120):
        L, S = int(rng.integers(1, 7)), int(rng.integers(1, 7))
        B = int(rng.integers(0, 65))
        tau, err, _ = workloads.random_instance(rng, 1, L, S, B, tau_max=int(rng.integers(1, 30)))
        p, c = oracle.solve_ref(tau, err, B)
        bp, bc, bt, nb = oracle.brute_force(tau, err, B)
        assert c[0].tobytes() == bc.tobytes()
        if bt < 0:
            assert (p[0] == -1).all() and np.isinf(c[0])
            continue
        assert profile_time(tau, p[0]) == bt
        assert fp32_sum_in_layer_order(err[0], p[0]).tobytes() == bc.tobytes()
        if nb == 1:
            n_unique += 1
            assert p[0].tolist() == bp.tolist()
    assert n_unique > 60


@pytest.mark.parametrize("seed", range(6))
def test_integer_errors_pin_both_tie_breaks(seed):
    """Small integer errors: all sums exact, ties everywhere.  The oracle must return the
    optimal profile that is smallest under (cost, total time, s_L, s_{L-1}, .., s_1), which is
    what "smallest level wins a cell" plus "smallest t wins the final argmin" imply.  Budgets are
    drawn around the middle of the reachable times, so that they bind (with a slack budget two
    tied profiles that differ in several layers always have a tied mixture that both ways of
    reading the key agree on)."""
    rng = np.random.default_rng(200 + seed)
    n_tied = 0
    for _ in range(120):
        L, S = int(rng.integers(1, 7)), int(rng.integers(2, 7))
        tau, err, _ = workloads.random_instance(rng, 1, L, S, 10 ** 6,
                                                tau_max=int(rng.integers(1, 12)),
                                                integer_err=int(rng.integers(1, 4)))
        lo, hi = int(tau.min(axis=1).sum()), int(tau.max(axis=1).sum())
        B = int(rng.integers(lo, max(lo, (lo + hi) // 2) + 1))
        p, c = oracle.solve_ref(tau, err, B)
        bp, bc, bt, nb = oracle.brute_force(tau, err, B)
        assert c[0].tobytes() == bc.tobytes()
        assert p[0].tolist() == bp.tolist()
        n_tied += nb > 1
    assert n_tied > 40


def load_golden_instances(path):
    """Several instances per file: "instance NAME" starts one; case rows carry the number of tied
    profiles before the levels."""
    out, cur = [], None
    with open(path) as f:
        for line in f:
            tok = line.split("#", 1)[0].split()
            if not tok:
                continue
            if tok[0] == "instance":
                cur = {"name": tok[1], "tau": [], "err": [], "cases": []}
                out.append(cur)
            elif tok[0] == "dims":
                cur["dims"] = (int(tok[1]), int(tok[2]))
            elif tok[0] == "tau":
                cur["tau"].append([int(x) for x in tok[1:]])
            elif tok[0] == "err":
                cur["err"].append([float(x) for x in tok[1:]])
            elif tok[0] == "case":
                cur["cases"].append((int(tok[1]), float(tok[2]), int(tok[3]), int(tok[4]),
                                     [int(x) for x in tok[5:]]))
    for inst in out:
        inst["tau"] = np.array(inst["tau"], dtype=np.int32)
        inst["err"] = np.array(inst["err"], dtype=np.float32)
        assert inst["tau"].shape == inst["dims"] and inst["err"].shape == inst["dims"]
    return out


def test_tied_optima_under_a_binding_budget(golden_dir):
    """Hand-worked instances whose optimum is attained by several profiles that differ in two or
    more layers while the budget binds: the dynamic program and the enumerator must both return
    the tied profile that is smallest read from the LAST layer down (strict "<" per cell, walk
    back from the last layer), which differs from the one smallest read from the first layer."""
    instances = load_golden_instances(os.path.join(golden_dir, "tied_optima_binding_budget.txt"))
    assert len(instances) >= 6
    separating = 0
    for inst in instances:
        tau, err = inst["tau"], inst["err"]
        for B, cost, t, n_tied, prof in inst["cases"]:
            p, c = oracle.solve_ref(tau, err, B)
            assert c[0] == F32(cost), (inst["name"], B, c)
            assert p[0].tolist() == prof, (inst["name"], B, p)
            bp, bc, bt, nb = oracle.brute_force(tau, err, B)
            assert bc == F32(cost) and bt == t and nb == n_tied, (inst["name"], B, bc, bt, nb)
            assert bp.tolist() == prof, (inst["name"], B, bp)
            # the fixture itself against a plain enumeration written here
            ec, et, winners = python_enumeration(tau, err, B)
            assert len(winners) == n_tied and et == t
            if winners:
                assert tuple(prof) == min(winners, key=lambda q: tuple(reversed(q)))
                separating += tuple(prof) != min(winners)
    assert separating >= 12


@pytest.mark.parametrize("seed", range(4))
def test_tie_key_reads_from_the_last_layer(seed):
    """Random small instances whose layers come in one or two KINDS (layers of a kind share their
    times and errors, like the repeated blocks of a network), integer errors, binding budgets:
    exchanging the levels of two layers of a kind keeps error and time, so tied optima that differ
    in several layers are the rule.  Winners are listed by a plain Python enumeration; both the
    dynamic program and the C enumerator must return the winner that is smallest read from the
    last layer down, on many instances where reading from the first layer up picks another."""
    rng = np.random.default_rng(900 + seed)
    separating = 0
    for _ in range(150):
        L, S = int(rng.integers(2, 5)), int(rng.integers(2, 4))
        kinds = int(rng.integers(1, 3))
        tau_k, err_k, _ = workloads.random_instance(rng, 1, kinds, S, 10 ** 6,
                                                    tau_max=int(rng.integers(1, 6)),
                                                    integer_err=int(rng.integers(2, 4)))
        kind = rng.integers(0, kinds, size=L)
        tau = np.ascontiguousarray(tau_k[kind])
        err = np.ascontiguousarray(err_k[:, kind])
        lo, hi = int(tau.min(axis=1).sum()), int(tau.max(axis=1).sum())
        B = int(rng.integers(lo, max(lo, (lo + hi) // 2) + 1))
        cost, t, winners = python_enumeration(tau, err[0], B)
        assert winners
        want = min(winners, key=lambda q: tuple(reversed(q)))
        p, c = oracle.solve_ref(tau, err, B)
        bp, bc, bt, nb = oracle.brute_force(tau, err, B)
        assert tuple(p[0].tolist()) == want and tuple(bp.tolist()) == want
        assert c[0] == F32(cost) and bc == F32(cost) and bt == t and nb == len(winners)
        separating += want != min(winners)
    assert separating >= 6, separating


def test_zero_times_over_budget_times_forbidden_levels_infeasible():
    """tau = 0 entries (a zero-time prefix must be extendable), tau > B entries, err = +inf
    entries and budgets nobody meets."""
    rng = np.random.default_rng(7)
    seen_infeasible = seen_zero_prefix = 0
    for trial in range(300):
        L, S = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        B = int(rng.integers(0, 25))
        tau, err, _ = workloads.random_instance(
            rng, 1, L, S, B, tau_max=10, integer_err=3 if trial % 2 else None,
            zero_tau_frac=0.35, over_budget_frac=0.15, inf_err_frac=0.1)
        p, c = oracle.solve_ref(tau, err, B)
        bp, bc, bt, nb = oracle.brute_force(tau, err, B)
        assert c[0].tobytes() == bc.tobytes()
        if bt < 0:
            seen_infeasible += 1
            assert (p[0] == -1).all()
            continue
        assert profile_time(tau, p[0]) == bt
        if trial % 2 or nb == 1:
            assert p[0].tolist() == bp.tolist()
        if L > 1 and tau[0, p[0][0]] == 0:
            seen_zero_prefix += 1
    assert seen_infeasible > 5 and seen_zero_prefix > 20


def test_all_zero_times_first_layer_zero_budget():
    """B = 0 with zero-time levels everywhere: only D[.][0] exists and must be usable."""
    tau = np.zeros((4, 3), dtype=np.int32)
    err = np.array([[[3, 1, 2], [5, 5, 4], [0, 7, 0], [2, 2, 2]]], dtype=np.float32)
    p, c = oracle.solve_ref(tau, err, 0)
    assert p[0].tolist() == [1, 2, 0, 0] and c[0] == F32(7)


# --------------------------------------------------------------------------- closed forms
def test_single_level_is_forced():
    rng = np.random.default_rng(3)
    L = 9
    tau = rng.integers(0, 6, size=(L, 1)).astype(np.int32)
    err = rng.random((2, L, 1), dtype=np.float32)
    T = int(tau.sum())
    p, c = oracle.solve_ref(tau, err, T)
    assert (p == 0).all()
    for k in range(2):
        assert c[k].tobytes() == fp32_sum_in_layer_order(err[k], [0] * L).tobytes()
    p, c = oracle.solve_ref(tau, err, T - 1)
    assert (p == -1).all() and np.isinf(c).all()


def test_single_layer_is_a_filtered_min():
    rng = np.random.default_rng(4)
    for _ in range(50):
        S, B = int(rng.integers(1, 9)), int(rng.integers(0, 12))
        tau = rng.integers(0, 15, size=(1, S)).astype(np.int32)
        err = rng.integers(0, 4, size=(1, 1, S)).astype(np.float32)
        p, c = oracle.solve_ref(tau, err, B)
        ok = [(float(err[0, 0, s]), int(tau[0, s]), s) for s in range(S) if tau[0, s] <= B]
        if not ok:
            assert p[0, 0] == -1 and np.isinf(c[0])
        else:
            e, _, s = min(ok)
            assert p[0, 0] == s and c[0] == F32(e)


def test_all_times_zero_is_per_layer_argmin():
    rng = np.random.default_rng(5)
    L, S = 7, 6
    tau = np.zeros((L, S), dtype=np.int32)
    err = rng.integers(0, 3, size=(3, L, S)).astype(np.float32)
    p, c = oracle.solve_ref(tau, err, 5)
    assert (p == err.argmin(axis=2)).all()          # numpy argmin = first occurrence
    assert (c == err.min(axis=2).sum(axis=1)).all()


def classic_knapsack(weights, values, cap):
    best = [0] * (cap + 1)
    for w, v in zip(weights, values):
        for c in range(cap, w - 1, -1):
            best[c] = max(best[c], best[c - w] + v)
    return best[cap]


def test_zero_one_knapsack_reduction():
    """S = 2: level 0 "take" (time w_l, error 0), level 1 "skip" (time 0, error v_l).
    Then optimum = sum(v) - (textbook 0/1 knapsack value at capacity B)."""
    rng = np.random.default_rng(6)
    for _ in range(60):
        L = int(rng.integers(1, 14))
        w = rng.integers(1, 20, size=L)
        v = rng.integers(0, 30, size=L)
        B = int(rng.integers(0, 60))
        tau = np.stack([w, np.zeros(L, dtype=np.int64)], axis=1).astype(np.int32)
        err = np.stack([np.zeros(L), v], axis=1).astype(np.float32)[None]
        p, c = oracle.solve_ref(tau, err, B)
        assert c[0] == F32(v.sum() - classic_knapsack(w.tolist(), v.tolist(), B))
        taken = p[0] == 0
        assert w[taken].sum() <= B and v[~taken].sum() == c[0]


def test_integer_program_cross_check():
    """Eq. 1 is an integer linear program (Sec. 3.1); solve small ones with scipy's MILP."""
    milp = pytest.importorskip("scipy.optimize").milp
    from scipy.optimize import Bounds, LinearConstraint
    rng = np.random.default_rng(8)
    for _ in range(25):
        L, S, B = int(rng.integers(2, 7)), int(rng.integers(2, 6)), int(rng.integers(5, 60))
        tau, err, _ = workloads.random_instance(rng, 1, L, S, B, tau_max=20, integer_err=9)
        n = L * S
        pick_one = np.zeros((L, n))
        for l in range(L):
            pick_one[l, l * S:(l + 1) * S] = 1
        res = milp(err[0].reshape(-1).astype(np.float64),
                   constraints=[LinearConstraint(pick_one, 1, 1),
                                LinearConstraint(tau.reshape(1, -1).astype(np.float64), -np.inf, B)],
                   integrality=np.ones(n), bounds=Bounds(0, 1))
        p, c = oracle.solve_ref(tau, err, B)
        if res.status == 2:       # infeasible
            assert np.isinf(c[0])
        else:
            assert res.status == 0
            assert c[0] == F32(round(res.fun))


# --------------------------------------------------------------------------- invariants
@pytest.mark.parametrize("name", ["tiny", "rn50_k1", "paper_rn50_k1024", "rn50_params_k1024"])
def test_invariants_on_benchmark_shaped_tables(name):
    cfg = workloads.CONFIGS[name]
    tau, err, B = workloads.generate(cfg, K=3)
    p, c = oracle.solve_ref(tau, err, B)
    L = cfg.L
    for k in range(3):
        # budget met, cost is the layer-order fp32 sum of the returned profile
        assert profile_time(tau, p[k]) <= B
        assert fp32_sum_in_layer_order(err[k], p[k]).tobytes() == c[k].tobytes()
        # batch independence
        p1, c1 = oracle.solve_ref(tau, err[k:k + 1], B)
        assert (p1[0] == p[k]).all() and c1[0].tobytes() == c[k].tobytes()
    # optimal cost never increases with the budget; the rows of D do not depend on B, so a
    # smaller budget is the same instance cut at t <= B'
    D, P, pk, ck = oracle.tables_ref(tau, err[0], B)
    assert (pk == p[0]).all() and ck.tobytes() == c[0].tobytes()
    last = D[L - 1]
    prev_cost = None
    for Bp in sorted({0, B // 7, B // 3, B // 2, (2 * B) // 3, B - 1, B}):
        pp, cp = oracle.solve_ref(tau, err[0], Bp)
        want = last[:Bp + 1].min()
        assert cp[0].tobytes() == F32(want).tobytes()
        if np.isfinite(want):
            assert profile_time(tau, pp[0]) == int(np.argmin(last[:Bp + 1]))
        if prev_cost is not None:
            assert cp[0] <= prev_cost
        prev_cost = cp[0]
    # dense profile (level 0 everywhere, cost 0) once the budget covers the dense model
    dense = int(tau[:, 0].sum())
    pd, cd = oracle.solve_ref(tau, err[0], dense)
    assert (pd[0] == 0).all() and cd[0] == 0
    pd, cd = oracle.solve_ref(tau, err[0], dense - 1)
    assert cd[0] > 0 and (pd[0] != 0).any()
    # scaling all errors by a power of two scales the cost exactly and keeps the profile
    for j in (-3, 5):
        ps, cs = oracle.solve_ref(tau, err[0] * F32(2.0 ** j), B)
        assert (ps[0] == p[0]).all() and cs[0] == c[0] * F32(2.0 ** j)


def test_matrices_are_consistent_with_the_recursion():
    """Every finite D[l][t] equals D[l-1][t - tau[l][P]] + err[l][P] bit for bit, and no level
    gives a strictly smaller value (Eq. 2), and among equal values P is the smallest level."""
    rng = np.random.default_rng(9)
    tau, err, B = workloads.random_instance(rng, 1, 6, 5, 40, tau_max=9, integer_err=3,
                                            zero_tau_frac=0.1)
    D, P, _, _ = oracle.tables_ref(tau, err[0], B)
    L, S = tau.shape
    for l in range(L):
        for t in range(B + 1):
            vals = []
            for s in range(S):
                u = t - int(tau[l, s])
                if u < 0:
                    vals.append(np.inf)
                elif l == 0:
                    vals.append(float(err[0, l, s]) if u == 0 else np.inf)
                else:
                    vals.append(float(F32(D[l - 1, u] + err[0, l, s])))
            m = min(vals)
            assert D[l, t] == F32(m)
            if np.isfinite(m):
                assert P[l, t] == vals.index(m)
            else:
                assert P[l, t] == -1


def test_subnormal_errors_are_kept():
    tiny = np.float32(1e-45)  # smallest fp32 subnormal
    tau = np.array([[1, 0], [1, 0]], dtype=np.int32)
    err = np.array([[[0, tiny], [0, tiny]]], dtype=np.float32)
    p, c = oracle.solve_ref(tau, err, 1)
    assert c[0] == tiny and c[0] > 0
    p, c = oracle.solve_ref(tau, err, 0)
    assert c[0] == F32(2) * tiny and p[0].tolist() == [1, 1]


def test_sensitivity_form_equals_the_explicit_table():
    """Eq. 4: err = c_l * w_s.  The fused routine must equal Alg. 1 on the table NumPy forms with
    its own fp32 multiply (one rounding of the exact product), including products that round."""
    rng = np.random.default_rng(12)
    for _ in range(30):
        K, L, S = int(rng.integers(1, 4)), int(rng.integers(1, 7)), int(rng.integers(2, 9))
        B = int(rng.integers(5, 80))
        tau, _, _ = workloads.random_instance(rng, 1, L, S, B, tau_max=25)
        c = rng.random((K, L), dtype=np.float32)
        w = np.square(np.arange(S, dtype=np.float64) / (S - 1)).astype(np.float32)   # Eq. 4
        err = (c[:, :, None] * w[None, None, :]).astype(np.float32)
        assert (err != (c[:, :, None].astype(np.float64) * w).astype(np.float32)).sum() == 0
        p1, c1 = oracle.solve_sens_ref(tau, c, w, B)
        p2, c2 = oracle.solve_ref(tau, err, B)
        assert (p1 == p2).all() and c1.tobytes() == c2.tobytes()
    # a product that is inexact in fp32 and would differ if it were kept in double
    tau = np.array([[1, 0]], dtype=np.int32)
    c = np.array([[F32(1) / F32(3)]], dtype=np.float32)
    w = np.array([F32(0.1), F32(0.7)], dtype=np.float32)
    p, cost = oracle.solve_sens_ref(tau, c, w, 0)
    assert cost[0].tobytes() == F32(c[0, 0] * w[1]).tobytes() and p[0, 0] == 1


# --------------------------------------------------------------------------- argument checks
def test_oracle_rejects_bad_inputs():
    tau = np.array([[1, 2]], dtype=np.int32)
    err = np.zeros((1, 1, 2), dtype=np.float32)
    assert oracle.solve_ref_status(tau, err, 3)[0] == 0
    assert oracle.solve_ref_status(tau, err, -1)[0] == -2
    bad = tau.copy()
    bad[0, 1] = -1
    assert oracle.solve_ref_status(bad, err, 3)[0] == -6
    for v in (np.nan, -np.inf):
        e = err.copy()
        e[0, 0, 0] = v
        assert oracle.solve_ref_status(tau, e, 3)[0] == -7
    e = err.copy()
    e[0, 0, 0] = np.inf            # +inf is a legal "forbidden level"
    st, p, c = oracle.solve_ref_status(tau, e, 3)
    assert st == 0 and p[0, 0] == 1


# --------------------------------------------------------------------------- work count
def test_resnet50_sized_solve_is_fast():
    """Sec. 3.2 quotes under 100 ms on a CPU for T = 10^4, |S| = 42, L = 52; a plain C loop nest
    of L*|S|*T updates should be well inside that (loose bound to stay robust on a busy host)."""
    rng = np.random.default_rng(0)
    tau, err, B = workloads.random_instance(rng, 1, 52, 42, 10000, tau_max=1500)
    oracle.solve_ref(tau, err, B)
    t0 = time.perf_counter()
    oracle.solve_ref(tau, err, B)
    dt = time.perf_counter() - t0
    assert dt < 0.5, dt


def test_threaded_runner_equals_serial():
    cfg = workloads.CONFIGS["tiny"]
    tau, err, B = workloads.generate(cfg, K=13)
    p1, c1 = oracle.solve_ref(tau, err, B, threads=1)
    p4, c4 = oracle.solve_ref(tau, err, B, threads=4)
    assert (p1 == p4).all() and c1.tobytes() == c4.tobytes()


# ------------------------------------------------------------------------------------------------
# Facts about fp32 arithmetic and about Alg. 1 that the device design leans on; checked here on
# the CPU with NumPy's IEEE fp32 and the oracle, so a violation shows up without a GPU.

def test_rounded_add_is_monotone_so_equal_time_levels_fold():
    """min_s fl(p + e_s) == fl(p + min_s e_s): levels of a layer that take the same time read the
    same cell p of D_{l-1}, so one update with their smallest error serves them all."""
    rng = np.random.default_rng(123)
    scales = [2.0 ** k for k in (-149, -140, -126, -30, -1, 0, 10, 60, 120)]
    for _ in range(400):
        p = F32(rng.random() * rng.choice(scales))
        if rng.random() < 0.1:
            p = F32(np.inf)
        e = (rng.random(7) * rng.choice(scales)).astype(F32)
        if rng.random() < 0.3:
            e[rng.integers(0, 7)] = F32(np.inf)
        if rng.random() < 0.3:
            e = np.where(np.isfinite(e), -e, e).astype(F32)   # negative finite errors are allowed
        with np.errstate(over="ignore"):
            each = np.array([F32(p + x) for x in e], dtype=F32)
            folded = F32(p + e.min())
        assert each.min() == folded                        # == : the sign of a zero may differ
    # and adjacent fp32 values: the add cannot reorder them
    x = F32(1.0)
    for e_lo in (F32(2.0 ** -24), F32(2.0 ** -25), F32(0.0)):
        e_hi = np.nextafter(e_lo, F32(1.0), dtype=F32)
        assert F32(x + e_lo) <= F32(x + e_hi)


def test_equal_time_levels_can_be_folded_in_alg1():
    """Replacing the levels of one time by a single level carrying their smallest error changes
    neither the optimal cost nor D anywhere (checked on the oracle's matrices)."""
    rng = np.random.default_rng(5)
    for _ in range(20):
        L, S, B = 5, 8, 60
        tau = rng.integers(0, 9, size=(L, S)).astype(np.int32)      # many equal times
        err = rng.random((1, L, S)).astype(F32)
        D, _, _, cost = oracle.tables_ref(tau, err, B)
        tau2 = np.full_like(tau, B + 1)                              # unused slots never fit
        err2 = np.full_like(err, np.inf)
        for l in range(L):
            for i, t in enumerate(np.unique(tau[l])):
                tau2[l, i] = t
                err2[0, l, i] = err[0, l][tau[l] == t].min()
        D2, _, _, cost2 = oracle.tables_ref(tau2, err2, B)
        assert np.array_equal(D, D2) and F32(cost) == F32(cost2)


def test_rows_do_not_depend_on_later_layers():
    """D_l is a function of layers 0..l only (Eq. 2): what lets a candidate that shares its first
    layers with a solved one start from that one's row."""
    rng = np.random.default_rng(6)
    tau, err, B = workloads.random_instance(rng, 1, 7, 6, 90, integer_err=4)
    D, _, _, _ = oracle.tables_ref(tau, err, B)
    other = err.copy()
    other[0, 4:] = rng.random((3, 6)).astype(F32)
    D2, _, _, _ = oracle.tables_ref(tau, other, B)
    assert np.array_equal(D[:4], D2[:4]) and not np.array_equal(D[4:], D2[4:])


def test_reduced_table_equals_alg1_on_the_cells_that_matter():
    """The exact reductions the device design rests on, replayed in NumPy against the oracle's
    matrix: subtract each layer's smallest time m_l (budget B - M, row l shifted by m_0 + .. + m_l),
    cut rows at the largest reachable reduced time, fold levels of equal time.  Every reduced cell
    must equal Alg. 1's D at the shifted time, cells beyond the reach bound must be +inf there, and
    the final argmin must pick the same (cost, t)."""
    rng = np.random.default_rng(99)
    for case in range(25):
        L, S = int(rng.integers(1, 7)), int(rng.integers(1, 9))
        B = int(rng.integers(0, 120))
        tau, err, _ = workloads.random_instance(
            rng, 1, L, S, B, tau_max=max(1, B // 2), integer_err=3 if case % 3 == 0 else None,
            zero_tau_frac=0.15, over_budget_frac=0.1, layer_floor=B // (2 * L) if case % 2 else 0)
        D, _, _, cost = oracle.tables_ref(tau, err, B)
        m = tau.min(axis=1).astype(np.int64)
        bp = B - int(m.sum())
        if bp < 0:
            assert np.isinf(cost)
            continue
        lo = np.cumsum(m)
        prev = np.full(bp + 1, np.inf, dtype=F32)
        prev[0] = F32(-0.0)                       # D before the first layer: time 0 costs nothing
        reach = 0
        for l in range(L):
            shift = tau[l].astype(np.int64) - m[l]
            usable = shift[shift <= bp]
            reach = min(reach + int(usable.max()), bp)
            cur = np.full(bp + 1, np.inf, dtype=F32)
            for d in np.unique(usable):           # one update per distinct time, smallest error
                e = err[0, l][shift == d].min()
                with np.errstate(invalid="ignore"):
                    cand = (prev[:bp + 1 - d] + e).astype(F32)
                cur[d:] = np.minimum(cur[d:], cand)
            assert np.isinf(cur[reach + 1:]).all()
            want = D[l, lo[l]:lo[l] + bp + 1]
            assert np.array_equal(cur, want), f"case {case} layer {l}"
            assert np.isinf(D[l, :lo[l]]).all()   # below the shifted origin nothing is reachable
            prev = cur
        t_red = int(np.argmin(prev))
        assert F32(prev[t_red]) == F32(cost) or (np.isinf(cost) and np.isinf(prev[t_red]))
        if np.isfinite(cost):
            assert t_red + int(m.sum()) == int(np.argmin(D[L - 1]))


def test_levels_that_cannot_win_may_be_left_out():
    """Alg. 1 with the levels in index order and strict "<", but leaving out every level for
    which an earlier level of the layer takes the same time with an error no larger: D and P must
    equal the oracle's everywhere D is finite (what the level-recording device sweep does)."""
    rng = np.random.default_rng(41)
    skipped = 0
    for case in range(30):
        L, S, B = int(rng.integers(1, 6)), int(rng.integers(2, 10)), int(rng.integers(5, 80))
        tau = rng.integers(0, 7, size=(L, S)).astype(np.int32)      # many equal times
        if case % 2:
            err = rng.integers(0, 3, size=(1, L, S)).astype(F32)     # equal errors too
        else:
            err = rng.random((1, L, S)).astype(F32)
        D_ref, P_ref, _, _ = oracle.tables_ref(tau, err, B)
        prev = np.full(B + 1, np.inf, dtype=F32)
        prev[0] = F32(-0.0)
        for l in range(L):
            cur = np.full(B + 1, np.inf, dtype=F32)
            arg = np.full(B + 1, -1, dtype=np.int64)
            for s in range(S):
                d = int(tau[l, s])
                if d > B:
                    continue
                if any(tau[l, q] == d and err[0, l, q] <= err[0, l, s] for q in range(s)):
                    skipped += 1
                    continue
                cand = (prev[:B + 1 - d] + err[0, l, s]).astype(F32)
                better = cand < cur[d:]
                cur[d:][better] = cand[better]
                arg[d:][better] = s
            fin = np.isfinite(D_ref[l])
            assert np.array_equal(cur, D_ref[l]), f"case {case} layer {l}"
            assert np.array_equal(arg[fin], P_ref[l][fin]), f"case {case} layer {l}"
            prev = cur
    assert skipped > 50
