"""GPU parity: the HIP path against the CPU oracle, bit for bit (profiles, fp32 costs, and the
per-cell level record wherever the oracle's D is finite), through the C-ABI binding."""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
CPU_THREADS = 16


@pytest.fixture(scope="module")
def dp():
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2201_13096_amd as m
    m.binding.lib()  # fails loudly if the HIP library was not built
    return m


@pytest.fixture(scope="module")
def reference():
    cache = {}

    def get(name, tau, err, B):
        if name not in cache:
            print(f"[parity] {name}: running the oracle on {CPU_THREADS} threads", flush=True)
            cache[name] = oracle.solve_ref(tau, err, B, threads=CPU_THREADS)
        return cache[name]
    return get


def gpu_solve(dp, tau, err, B, compact=False, stream=None):
    dev = torch.device("cuda:0")
    tau_d = torch.from_numpy(tau).to(dev)
    err_d = torch.from_numpy(err).to(dev)
    K, L, S = err.shape
    ws = dp.alloc_workspace(K, L, S, B, dev, compact=compact)
    if ws.numel() < 2 ** 31:
        ws.fill_(0xAB)   # stale contents must not matter
    profile = torch.full((K, L), -7, dtype=torch.int16, device=dev)
    cost = torch.full((K,), -7.0, dtype=torch.float32, device=dev)
    dp.spdy_dp_solve_batched(tau_d, err_d, B, profile, cost, ws, stream=stream)
    torch.cuda.synchronize()
    return profile.cpu().numpy(), cost.cpu().numpy(), ws


def assert_same(p_gpu, c_gpu, p_ref, c_ref, what):
    bad_c = np.flatnonzero(c_gpu.view(np.uint32) != c_ref.view(np.uint32))
    assert bad_c.size == 0, f"{what}: cost bits differ at candidates {bad_c[:8]}: " \
                            f"{c_gpu[bad_c[:8]]} vs {c_ref[bad_c[:8]]}"
    bad_p = np.argwhere(p_gpu != p_ref)
    assert bad_p.size == 0, f"{what}: profiles differ at (k, l) {bad_p[:8].tolist()}"


def check_tables(dp, tau, err_k, B, ws, k, K):
    """The record of candidate k against the oracle's matrices.  The device works on reduced
    times t' = t - (m_0 + .. + m_l) with m_l = min_s tau[l][s] and computes only chunks that can
    be finite; every computed cell must equal the oracle's D (value record) or P (level record,
    where D is finite), every cell it skips must be +inf in the oracle, and t* must agree."""
    L, S = tau.shape
    D, P, prof, cost = oracle.tables_ref(tau, err_k, B)
    lay = dp.spdy_dp_workspace_layout(K, L, S, B, ws.numel())
    H, plan = lay["header_words"], lay["plan_words"]
    meta = ws[lay["meta_offset"]:lay["meta_offset"] + 4 * (H + (3 + plan) * L)].cpu().numpy() \
        .view(np.int32)
    mn = tau.min(axis=1).astype(np.int64)
    M = int(mn.sum())
    tstar = ws[lay["tstar_offset"] + 4 * k:lay["tstar_offset"] + 4 * k + 4].cpu().numpy() \
        .view(np.int32)[0]
    if M > B:
        assert meta[0] == -1 and tstar == -1 and np.isinf(cost)
        return
    bp = B - M
    assert meta[0] == bp and meta[1] == M and meta[2] == (bp + 64) // 64 * 64
    assert (meta[H:H + L] == mn).all()
    nact = meta[H + L:H + 2 * L].astype(np.int64)
    # the largest usable shift of each layer (what a staged tile of the global-row path reaches)
    delta = tau.astype(np.int64) - mn[:, None]
    assert (meta[H + (2 + plan) * L:H + (3 + plan) * L] ==
            np.where(delta <= bp, delta, 0).max(axis=1)).all()
    lo = np.cumsum(mn)
    pitch, rows = lay["record_pitch"], lay["record_rows"]
    esize = 4 if lay["variant"] == 0 else 1
    a = lay["record_offset"] + k * rows * pitch * esize
    rec = ws[a:a + rows * pitch * esize].cpu().numpy()
    rec = rec.view(np.float32 if esize == 4 else np.uint8).reshape(rows, pitch)
    # Which launch did the work must follow from what the header says the choice was made from
    # (no tuning constant is repeated here): a row is updated in place exactly when the waves of
    # a workgroup can hold all its chunks in registers (the usual workgroup, or, for the D
    # record, the wide one with a compute unit's LDS to itself); otherwise two rows (with their
    # aprons) alternate in LDS if the larger launch has room for them, else they live in global
    # memory.
    path, team_waves, teams, inplace = (int(x) for x in meta[3:7])
    waves, max_group, lds_small, lds_large, halo, split, wide_waves, wide_group, lds_wide, \
        global_waves = (int(x) for x in meta[8:18])
    # a D-record candidate with at most 64 levels that has a compute unit to itself is swept by
    # twice the planned waves (the plan itself is the same)
    units = torch.cuda.get_device_properties(0).multi_processor_count
    assert split == int(K <= units and lay["variant"] == 0 and S <= 64)
    chunks = int(meta[2]) // 64
    row_bytes = (int(meta[2]) + halo) * 4
    fits_place = chunks <= waves * max_group
    fits_wide = wide_waves > 0 and chunks <= wide_waves * wide_group and row_bytes <= lds_wide
    assert inplace == int(fits_place or fits_wide)
    assert wide_waves == 0 or (lay["variant"] == 0 and lds_large == 0)
    if fits_place:
        assert path == 1 and row_bytes * teams <= lds_small
        assert 1 <= teams and teams * team_waves <= waves
        assert chunks <= team_waves * max_group         # a team's waves hold the whole row
    elif fits_wide:
        assert path == 3 and teams == 1 and team_waves == wide_waves
        max_group = wide_group
    elif 2 * row_bytes <= lds_large:
        assert path == 2 and teams == 1
    else:       # rows in global memory; twice the waves for the D record
        assert global_waves == (2 * waves if lay["variant"] == 0 else waves)
        assert path == (4 if global_waves > waves else 0) and teams == 1
        assert team_waves == global_waves
    # every wave's share of every row fits its registers when the row is updated in place
    plan_rows = meta[H + 2 * L:H + (2 + plan) * L].reshape(L, plan)[:, :team_waves + 1]
    assert (plan_rows[:, 0] == 0).all() and (plan_rows[:, team_waves] == nact).all()
    assert (np.diff(plan_rows, axis=1) >= 0).all()
    if inplace:
        assert (np.diff(plan_rows, axis=1) <= max_group).all()
    for l in range(L):
        n = int(min(nact[l] * 64, bp + 1))
        want_D = D[l, lo[l]:lo[l] + n]
        assert np.isinf(D[l, lo[l] + n:lo[l] + bp + 1]).all(), f"layer {l}: reach bound wrong"
        if lay["variant"] == 0:
            got = rec[l, :n]
            assert (got == want_D).all(), f"layer {l}: D record differs"
        else:
            fin = np.isfinite(want_D)
            got = rec[l, :n]
            assert (got[fin] == P[l, lo[l]:lo[l] + n][fin].astype(np.uint8)).all(), \
                f"layer {l}: level record differs"
    if np.isfinite(cost):
        assert tstar + M == int(np.argmin(D[L - 1]))
    else:
        assert tstar == -1


# --------------------------------------------------------------------------- the five configs
@pytest.mark.parametrize("compact", [False, True], ids=["d_record", "level_record"])
@pytest.mark.parametrize("name", ["tiny", "rn50_k1", "rn50_k1024", "bert_k4096", "stress_k256",
                                  "paper_rn50_k1024", "rn50_params_k1024"])
def test_config_bit_exact(dp, name, compact, reference):
    cfg = workloads.CONFIGS[name]
    print(f"[parity] config {name}: K={cfg.K} L={cfg.L} S={cfg.S} B={cfg.B} "
          f"compact={compact}", flush=True)
    tau, err, B = workloads.generate(cfg)
    p_gpu, c_gpu, ws = gpu_solve(dp, tau, err, B, compact=compact)
    print(f"[parity] {name}: gpu done", flush=True)
    p_ref, c_ref = reference(name, tau, err, B)
    assert_same(p_gpu, c_gpu, p_ref, c_ref, name)
    assert np.isfinite(c_ref).all()
    # properties that hold at any size: budget met; cost is the layer-order fp32 sum
    t = np.take_along_axis(np.broadcast_to(tau, err.shape), p_gpu[:, :, None].astype(np.int64),
                           axis=2)[:, :, 0].sum(axis=1)
    assert (t <= B).all()
    e = np.take_along_axis(err, p_gpu[:, :, None].astype(np.int64), axis=2)[:, :, 0]
    acc = e[:, 0].copy()
    for l in range(1, cfg.L):
        acc = (acc + e[:, l]).astype(np.float32)
    assert (acc.view(np.uint32) == c_gpu.view(np.uint32)).all()
    for k in sorted({0, cfg.K // 2, cfg.K - 1}):
        check_tables(dp, tau, err[k], B, ws, k, cfg.K)


@pytest.mark.parametrize("name", ["stress_x38_k256", "stress_x30_k256", "stress_x25_k256",
                                  "rn50_b100k_k1024", "rn50_s128_k1024"])
def test_long_row_workloads_on_sampled_candidates(dp, name):
    """The workloads that take the other launches of the fill (one long row in LDS swept by
    sixteen waves, rows in global memory, more than 64 levels), at the sizes their profiles are
    taken on: the whole batch is solved, sixteen candidates spread over it are compared with the
    oracle (one of them table by table), and the properties that need no oracle are checked on
    all of them."""
    cfg = workloads.CONFIGS[name]
    print(f"[parity] workload {name}: K={cfg.K} L={cfg.L} S={cfg.S} B={cfg.B}", flush=True)
    tau, err, B = workloads.generate(cfg)
    p_gpu, c_gpu, ws = gpu_solve(dp, tau, err, B)
    print(f"[parity] {name}: gpu done", flush=True)
    pick = np.unique(np.linspace(0, cfg.K - 1, 16).astype(np.int64))
    p_ref, c_ref = oracle.solve_ref(tau, np.ascontiguousarray(err[pick]), B, threads=CPU_THREADS)
    assert_same(p_gpu[pick], c_gpu[pick], p_ref, c_ref, name)
    t = np.take_along_axis(np.broadcast_to(tau, err.shape), p_gpu[:, :, None].astype(np.int64),
                           axis=2)[:, :, 0].sum(axis=1)
    assert (t <= B).all()
    e = np.take_along_axis(err, p_gpu[:, :, None].astype(np.int64), axis=2)[:, :, 0]
    acc = e[:, 0].copy()
    for l in range(1, cfg.L):
        acc = (acc + e[:, l]).astype(np.float32)
    assert (acc.view(np.uint32) == c_gpu.view(np.uint32)).all()
    check_tables(dp, tau, err[cfg.K - 1], B, ws, cfg.K - 1, cfg.K)


# --------------------------------------------------------------------------- shapes and edges
EDGE_SHAPES = [
    # K, L, S, B  (B + 1 deliberately not a multiple of 64 in most; several chunks per wave)
    (3, 1, 1, 0), (2, 1, 5, 7), (4, 5, 1, 100), (5, 6, 7, 63), (5, 6, 7, 64), (3, 9, 12, 1000),
    (7, 12, 33, 2500), (2, 4, 255, 700), (3, 17, 40, 10000), (2, 20, 16, 16384),
    (2, 7, 9, 17599), (2, 6, 10, 17600),             # around the largest rows two of which fit LDS
    (3, 6, 10, 20480),                               # one row in LDS, twice the waves
    (2, 5, 9, 26623), (2, 5, 9, 26624),              # around the longest row they keep in registers
    (300, 3, 5, 22000),                              # ... with more candidates than compute units
    (2, 5, 12, 33000), (1, 4, 6, 70001),             # rows in global memory, tiles
    (1, 2, 5, 70001),     # ... and shifts too long for a tile's window in LDS
    (300, 3, 5, 30000),   # ... and more candidates than compute units (level record: two
                          # workgroups per unit with half-size windows)
    (2, 300, 3, 500),                                # more layers than prepare threads
    (2, 5, 64, 300), (2, 5, 65, 300), (3, 4, 129, 900),       # level-block boundaries
    (2, 3, 70, 20480), (1, 3, 70, 40000),            # ... with long rows (LDS, global memory)
    (37, 4, 5, 200), (19, 3, 6, 1500),               # few candidates: one team per workgroup
    # more candidates than the chip holds at once: several teams per workgroup, the last
    # workgroup partly filled
    (1100, 4, 5, 700), (2600, 3, 6, 1500), (4100, 3, 4, 500),
    # one or two workgroups per compute unit: the instantiation whose workgroups take turns at
    # the instruction priority
    (300, 4, 5, 700), (700, 3, 6, 1500), (1024, 3, 4, 500),
]


@pytest.mark.parametrize("shape", EDGE_SHAPES)
def test_random_tables_bit_exact(dp, shape):
    K, L, S, B = shape
    print(f"[parity] random tables K={K} L={L} S={S} B={B}", flush=True)
    rng = np.random.default_rng(K * 1000003 + L * 10007 + S * 101 + B)
    for variant in range(7):
        kw = dict(tau_max=max(1, B // max(1, L // 2)))
        if variant == 1:
            kw.update(integer_err=3)                        # ties everywhere
        elif variant == 2:
            kw.update(zero_tau_frac=0.2, over_budget_frac=0.2, inf_err_frac=0.1)
        elif variant == 3:
            kw.update(integer_err=2, zero_tau_frac=0.3, tau_max=max(1, B // (2 * L) + 1))
        elif variant == 4:   # large per-layer floors: the reduced budget is a fraction of B
            kw.update(integer_err=4, tau_max=max(1, B // (2 * L)), layer_floor=B // L)
        elif variant == 5:   # errors in the fp32 subnormal range, some times at the int32 limit
            kw.update(err_scale=2.0 ** -140, huge_tau_frac=0.1)
        elif variant == 6:   # subnormal integers: ties and subnormals together
            kw.update(integer_err=5, err_scale=2.0 ** -149, zero_tau_frac=0.1)
        tau, err, _ = workloads.random_instance(rng, K, L, S, B, **kw)
        p_ref, c_ref = oracle.solve_ref(tau, err, B)
        for compact in (False, True):
            p_gpu, c_gpu, ws = gpu_solve(dp, tau, err, B, compact=compact)
            assert_same(p_gpu, c_gpu, p_ref, c_ref, f"{shape} variant {variant} compact={compact}")
            check_tables(dp, tau, err[K - 1], B, ws, K - 1, K)


def test_every_group_size_of_the_sweep(dp):
    """Row lengths chosen so that a wave's share of the row takes every size from one chunk up
    to the most a wave keeps in registers (the sweep is specialised per size: so many chunks
    read four buckets per lane, so many one), with one candidate per workgroup (eight waves on a
    row) and with several (teams of fewer waves), shifts of every residue mod 4 and layers whose
    shifts all share one residue.  Each of the three in-place launches sees every size: the one
    for candidates that have a compute unit to themselves (two waves per share of the row), the
    one for one or two rounds of workgroups, and the one for long batches."""
    rng = np.random.default_rng(4242)
    dev = torch.device("cuda:0")
    lay = dp.spdy_dp_workspace_layout(1, 2, 2, 64, dp.spdy_dp_workspace_bytes(1, 2, 2, 64))
    units = torch.cuda.get_device_properties(0).multi_processor_count
    long_batch = 4 * units + 70
    seen = {1: set(), 600: set(), long_batch: set()}
    for K in seen:
        sizes = list(range(1, 17)) + list(range(17, 8 * 28 + 1, 5)) + [8 * 28]
        if K == long_batch:       # every share from 1 to 26 chunks once, and two ragged rows
            sizes = [8 * r for r in range(1, 27)] + [13, 203]
        for chunks in sizes:
            B = 64 * chunks - int(rng.integers(1, 64))          # reduced row of `chunks` chunks
            L, S = 3, 7
            tau = rng.integers(0, max(2, B // 3), size=(L, S)).astype(np.int32)
            tau[:, 0] = 0                                       # m_l = 0: the row is not reduced
            tau[:, 1] = (B + 2) // 3 + 4                        # the last row is reached in full
            if chunks % 3 == 0:
                tau[1] = tau[1] // 4 * 4 + int(rng.integers(0, 4))   # one residue for a layer
                tau[1, 0] = 0
            kk = K
            err = rng.integers(0, 5, size=(kk, L, S)).astype(np.float32) if chunks % 2 else \
                rng.random((kk, L, S), dtype=np.float32)
            p_ref, c_ref = oracle.solve_ref(tau, err, B, threads=CPU_THREADS)
            p_gpu, c_gpu, ws = gpu_solve(dp, tau, err, B)
            assert_same(p_gpu, c_gpu, p_ref, c_ref, f"K={kk} chunks={chunks} B={B}")
            check_tables(dp, tau, err[kk - 1], B, ws, kk - 1, kk)
            H, plan = lay["header_words"], lay["plan_words"]
            off = dp.spdy_dp_workspace_layout(kk, L, S, B, ws.numel())["meta_offset"]
            meta = ws[off:off + 4 * (H + (3 + plan) * L)].cpu().numpy().view(np.int32)
            team_waves = int(meta[4])
            shares = meta[H + 2 * L:H + (2 + plan) * L].reshape(L, plan)[:, :team_waves + 1]
            seen[K].update(int(x) for x in np.diff(shares, axis=1).ravel())
            assert int(meta[13]) == int(kk <= units)
    for K, most in ((1, 26), (600, 28), (long_batch, 26)):
        assert set(range(1, most + 1)) <= seen[K], (K, sorted(set(range(1, most + 1)) - seen[K]))


def test_infeasible_and_mixed_batches(dp):
    # candidate 0 feasible, candidate 1 has every level of layer 2 forbidden, budget too small
    tau = np.array([[5, 3, 1], [4, 2, 1], [6, 2, 2]], dtype=np.int32)
    err = np.array([[[0, 1, 2], [0, 1, 2], [0, 1, 2]],
                    [[0, 1, 2], [0, 1, 2], [np.inf, np.inf, np.inf]]], dtype=np.float32)
    for B in (0, 3, 4, 9, 15, 200):
        p_ref, c_ref = oracle.solve_ref(tau, err, B)
        for compact in (False, True):
            p_gpu, c_gpu, _ = gpu_solve(dp, tau, err, B, compact=compact)
            assert_same(p_gpu, c_gpu, p_ref, c_ref, f"B={B} compact={compact}")
            assert np.isinf(c_gpu[1]) and (p_gpu[1] == -1).all()


def test_negative_zero_and_subnormal_errors(dp):
    tiny = np.float32(1e-45)
    tau = np.array([[1, 0], [1, 0], [2, 0]], dtype=np.int32)
    err = np.array([[[0, tiny], [0, tiny], [0, tiny]],
                    [[-0.0, 1], [-0.0, 1], [-0.0, 1]],
                    [[1, -0.0], [-0.0, 0.0], [0.0, -0.0]],
                    [[-1, 2], [3, -2.5], [0.5, -0.0]]], dtype=np.float32)
    for B in (0, 1, 2, 4, 70):
        p_ref, c_ref = oracle.solve_ref(tau, err, B)
        for compact in (False, True):
            p_gpu, c_gpu, _ = gpu_solve(dp, tau, err, B, compact=compact)
            assert_same(p_gpu, c_gpu, p_ref, c_ref, f"B={B} compact={compact}")


def test_stages_equal_the_fused_call_and_streams(dp):
    cfg = workloads.CONFIGS["rn50_k1"]
    tau, err, B = workloads.generate(cfg, K=5)
    dev = torch.device("cuda:0")
    tau_d, err_d = torch.from_numpy(tau).to(dev), torch.from_numpy(err).to(dev)
    K, L, S = err.shape
    ws = dp.alloc_workspace(K, L, S, B, dev)
    cost = torch.empty(K, dtype=torch.float32, device=dev)
    profile = torch.empty((K, L), dtype=torch.int16, device=dev)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        dp.spdy_dp_fill(tau_d, err_d, B, cost, ws)
        dp.spdy_dp_backtrace(tau_d, err_d, B, profile, cost, ws)
    side.synchronize()
    p_ref, c_ref = oracle.solve_ref(tau, err, B)
    assert_same(profile.cpu().numpy(), cost.cpu().numpy(), p_ref, c_ref, "staged, side stream")
    p2, c2, _ = gpu_solve(dp, tau, err, B)
    assert_same(p2, c2, p_ref, c_ref, "fused")


@pytest.mark.parametrize("compact", [False, True], ids=["d_record", "level_record"])
def test_sensitivity_form_bit_exact(dp, compact):
    """err = c_l * w_s formed on the device (Eq. 4) against the oracle's fused routine."""
    dev = torch.device("cuda:0")
    cases = []
    cfg = workloads.CONFIGS["paper_rn50_k1024"]
    tau, _, B = workloads.generate(cfg, K=1)
    rng = np.random.default_rng(5)
    w = np.square(np.arange(cfg.S, dtype=np.float64) / (cfg.S - 1)).astype(np.float32)
    cases.append((tau, rng.random((96, cfg.L), dtype=np.float32), w, B))
    for (K, L, S, B) in [(3, 4, 5, 90), (5, 9, 70, 1200), (2, 6, 130, 22000)]:
        tau, _, _ = workloads.random_instance(rng, 1, L, S, B, tau_max=max(1, B // L))
        cases.append((tau, rng.random((K, L), dtype=np.float32),
                      rng.random(S, dtype=np.float32), B))
    for tau, c, w, B in cases:
        K, L = c.shape
        S = w.shape[0]
        print(f"[parity] sensitivities K={K} L={L} S={S} B={B} compact={compact}", flush=True)
        ws = dp.alloc_workspace(K, L, S, B, dev, compact=compact)
        profile, cost = dp.spdy_dp_solve_sensitivities(
            torch.from_numpy(tau).to(dev), torch.from_numpy(c).to(dev),
            torch.from_numpy(w).to(dev), B, workspace=ws)
        torch.cuda.synchronize()
        p_ref, c_ref = oracle.solve_sens_ref(tau, c, w, B)
        assert_same(profile.cpu().numpy(), cost.cpu().numpy(), p_ref, c_ref, "sensitivities")


def test_several_budgets_from_one_fill(dp):
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(21)
    cfg = workloads.CONFIGS["rn50_k1"]
    tau, err, B = workloads.generate(cfg, K=24)
    dense = int(tau[:, 0].sum())
    fastest = int(tau.min(axis=1).sum())
    cases = [(tau, err, [B, B // 2, fastest, fastest - 1, 0, (3 * B) // 4, B, dense, dense + 7])]
    for (K, L, S, Bm) in [(3, 5, 6, 300), (4, 7, 70, 2500), (2, 6, 9, 30000)]:
        t, e, _ = workloads.random_instance(rng, K, L, S, Bm, tau_max=max(1, Bm // L),
                                            integer_err=3, zero_tau_frac=0.1, layer_floor=Bm // (3 * L))
        cases.append((t, e, [Bm, Bm // 3, 0, Bm - 1, int(t.min(axis=1).sum()), Bm // 2]))
    for tau, err, budgets in cases:
        print(f"[parity] budgets {budgets} K={err.shape[0]} L={err.shape[1]} S={err.shape[2]}",
              flush=True)
        profile, cost = dp.spdy_dp_solve_budgets(torch.from_numpy(tau).to(dev),
                                                 torch.from_numpy(err).to(dev), budgets)
        torch.cuda.synchronize()
        p_ref, c_ref = oracle.solve_budgets_ref(tau, err, budgets)
        for j, b in enumerate(budgets):
            assert_same(profile[j].cpu().numpy(), cost[j].cpu().numpy(), p_ref[j], c_ref[j],
                        f"budget {b}")
    # the level record does not keep the last row of D: a small workspace is refused
    K, L, S = cases[0][1].shape
    ws = dp.alloc_workspace(K, L, S, max(cases[0][2]), dev, compact=True)
    with pytest.raises(dp.SpdyDpError) as e:
        dp.spdy_dp_solve_budgets(torch.from_numpy(cases[0][0]).to(dev),
                                 torch.from_numpy(cases[0][1]).to(dev), cases[0][2], workspace=ws)
    assert e.value.status == -4


def mutate_from(rng, base, first_layer, err_draw):
    """Candidates that equal `base` [L, S] before first_layer[k] and differ (at that layer and at
    a random subset of the later ones) from it after."""
    K = first_layer.size
    L, S = base.shape
    err = np.repeat(base[None], K, axis=0)
    for k in range(K):
        f = int(np.clip(first_layer[k], 0, L))
        for l in range(f, L):
            if l == f or rng.random() < 0.3:
                err[k, l] = err_draw(l)
    return np.ascontiguousarray(err)


RESUME_SHAPES = [
    # (L, S, B, K, tau_max): rows in registers with teams, one team per workgroup, the large LDS
    # rows, the rows in global memory, and more than 64 levels
    (6, 5, 300, 37, None),
    (9, 8, 2000, 21, 400),
    (54, 40, 10000, 48, None),
    (12, 40, 30000, 9, 4000),
    (5, 12, 70000, 5, 20000),
    (7, 130, 5000, 11, 900),
    (6, 5, 300, 1300, None),     # more candidates than workgroup slots: teams with different starts
]


@pytest.mark.parametrize("shape", RESUME_SHAPES, ids=lambda s: "L%d_S%d_B%d_K%d" % s[:4])
def test_resume_from_incumbent_bit_exact(dp, shape):
    L, S, B, K, tau_max = shape
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(L * 1000 + S)
    if (L, S, B) == (54, 40, 10000):
        tau, base, _ = workloads.generate(workloads.CONFIGS["rn50_k1"], seed=5)
        w = np.square(workloads.level_grid(S, 0.9))
        draw = lambda l: (rng.random() * w).astype(np.float32)
    else:
        tau, base, _ = workloads.random_instance(rng, 1, L, S, B, tau_max=tau_max, integer_err=4,
                                                 zero_tau_frac=0.05, layer_floor=B // (4 * L))
        draw = lambda l: rng.integers(0, 4, size=S).astype(np.float32)
    first_layer = rng.integers(0, L + 1, size=K).astype(np.int32)
    first_layer[:4] = [0, L, 1, L - 1]
    first_layer[4] = -3          # clamped to 0
    err = mutate_from(rng, base[0], first_layer, draw)
    given = first_layer.copy()
    if K > 8:
        given[5] = L + 9         # clamped to L: candidate 5 must then equal the incumbent
        err[5] = base[0]
    print(f"[parity] resume L={L} S={S} B={B} K={K}", flush=True)
    tau_d = torch.from_numpy(tau).to(dev)
    inc_ws = dp.alloc_workspace(1, L, S, B, dev)
    inc_ws.fill_(0xAB)
    p_inc, c_inc = dp.spdy_dp_solve_batched(tau_d, torch.from_numpy(base).to(dev), B,
                                            workspace=inc_ws)
    ws = dp.alloc_workspace(K, L, S, B, dev)
    ws.fill_(0xCD)
    for order in ("given", "sorted"):
        idx = np.arange(K) if order == "given" else np.argsort(given, kind="stable")
        profile, cost = dp.spdy_dp_solve_from_incumbent(
            tau_d, torch.from_numpy(err[idx]).to(dev), torch.from_numpy(given[idx]).to(dev), B,
            inc_ws, workspace=ws)
        torch.cuda.synchronize()
        p_ref, c_ref = oracle.solve_ref(tau, err[idx], B, threads=CPU_THREADS)
        assert_same(profile.cpu().numpy(), cost.cpu().numpy(), p_ref, c_ref, f"resume {order}")
    # the incumbent's workspace was only read: solving from it again still works
    p_ref, c_ref = oracle.solve_ref(tau, base, B)
    assert_same(p_inc.cpu().numpy(), c_inc.cpu().numpy(), p_ref, c_ref, "incumbent")
    profile, cost = dp.spdy_dp_solve_from_incumbent(
        tau_d, torch.from_numpy(base).to(dev), torch.full((1,), L, dtype=torch.int32, device=dev),
        B, inc_ws)
    torch.cuda.synchronize()
    assert_same(profile.cpu().numpy(), cost.cpu().numpy(), p_ref, c_ref, "incumbent again")


def test_resume_from_an_infeasible_incumbent(dp):
    dev = torch.device("cuda:0")
    tau = np.array([[5, 6], [7, 9], [4, 4]], dtype=np.int32)
    base = np.array([[[1, 0], [2, 1], [0, 3]]], dtype=np.float32)
    for B in (15, 16, 17):       # the fastest profile takes 16
        tau_d = torch.from_numpy(tau).to(dev)
        inc_ws = dp.alloc_workspace(1, 3, 2, B, dev)
        dp.spdy_dp_solve_batched(tau_d, torch.from_numpy(base).to(dev), B, workspace=inc_ws)
        err = np.repeat(base, 4, axis=0)
        err[1, 2] = [5, 0]
        err[2, 1] = [0, 9]
        first = np.array([3, 2, 1, 0], dtype=np.int32)
        profile, cost = dp.spdy_dp_solve_from_incumbent(
            tau_d, torch.from_numpy(err).to(dev), torch.from_numpy(first).to(dev), B, inc_ws)
        torch.cuda.synchronize()
        p_ref, c_ref = oracle.solve_ref(tau, err, B)
        assert_same(profile.cpu().numpy(), cost.cpu().numpy(), p_ref, c_ref, f"B={B}")


CHECKPOINT_SHAPES = [
    # K, L, S, B, strides: teams in LDS, long rows in LDS, rows in global memory, S > 64, L = 1
    (37, 9, 8, 2000, (0, 1, 2, 4, 9, 50)),
    (5, 12, 40, 30000, (0, 5)),
    (3, 5, 12, 70000, (2,)),
    (7, 10, 130, 5000, (0, 3)),
    (4, 1, 6, 100, (0, 3)),
    (1300, 6, 5, 300, (0, 4)),
]


@pytest.mark.parametrize("shape", CHECKPOINT_SHAPES, ids=lambda s: "K%d_L%d_S%d_B%d" % s[:4])
def test_checkpointed_solve_bit_exact(dp, shape):
    K, L, S, B, strides = shape
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(K + 31 * L + 977 * S)
    for variant in range(3):
        kw = dict(tau_max=max(1, B // max(1, L // 2)))
        if variant == 1:
            kw.update(integer_err=3, zero_tau_frac=0.2)
        elif variant == 2:
            kw.update(over_budget_frac=0.3, inf_err_frac=0.1, layer_floor=B // L)
        tau, err, _ = workloads.random_instance(rng, K, L, S, B, **kw)
        if variant == 2:
            err[0, 0, :] = np.inf                 # candidate 0 has no feasible profile
        p_ref, c_ref = oracle.solve_ref(tau, err, B, threads=CPU_THREADS)
        for stride in strides:
            print(f"[parity] checkpointed K={K} L={L} S={S} B={B} stride={stride} v{variant}",
                  flush=True)
            n = dp.spdy_dp_workspace_bytes_checkpointed(K, L, S, B, stride)
            ws = torch.empty(n, dtype=torch.uint8, device=dev)
            ws.fill_(0xC3)
            profile = torch.full((K, L), -7, dtype=torch.int16, device=dev)
            cost = torch.full((K,), -7.0, dtype=torch.float32, device=dev)
            dp.spdy_dp_solve_checkpointed(torch.from_numpy(tau).to(dev),
                                          torch.from_numpy(err).to(dev), B, stride, profile, cost,
                                          ws)
            torch.cuda.synchronize()
            assert_same(profile.cpu().numpy(), cost.cpu().numpy(), p_ref, c_ref,
                        f"{shape[:4]} stride {stride} variant {variant}")


def test_checkpointed_solve_on_a_benchmark_shape(dp, reference):
    dev = torch.device("cuda:0")
    cfg = workloads.CONFIGS["rn50_k1024"]
    tau, err, B = workloads.generate(cfg)
    p_ref, c_ref = reference("rn50_k1024", tau, err, B)
    profile, cost = dp.spdy_dp_solve_checkpointed(torch.from_numpy(tau).to(dev),
                                                  torch.from_numpy(err).to(dev), B)
    torch.cuda.synchronize()
    assert_same(profile.cpu().numpy(), cost.cpu().numpy(), p_ref, c_ref, "rn50_k1024 checkpointed")


def test_many_random_shapes_through_every_entry_point(dp):
    """Seeded sweep over small random shapes: the plain solve with both records, the solve with
    checkpoints, several budgets and the sensitivity form, all against the oracle."""
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(2024)
    for case in range(40):
        K = int(rng.integers(1, 9))
        L = int(rng.integers(1, 12))
        S = int(rng.choice([1, 2, 3, 5, 8, 17, 40, 64, 65, 100]))
        B = int(rng.choice([0, 1, 7, 63, 64, 200, 1000, 5000]))
        kw = dict(tau_max=max(1, B // max(1, L // 2)), zero_tau_frac=float(rng.choice([0, 0.2])),
                  over_budget_frac=float(rng.choice([0, 0.1])),
                  integer_err=int(rng.choice([0, 2, 4])) or None)
        tau, err, _ = workloads.random_instance(rng, K, L, S, B, **kw)
        print(f"[parity] sweep {case}: K={K} L={L} S={S} B={B}", flush=True)
        p_ref, c_ref = oracle.solve_ref(tau, err, B)
        tau_d, err_d = torch.from_numpy(tau).to(dev), torch.from_numpy(err).to(dev)
        for compact in (False, True):
            p, c, _ = gpu_solve(dp, tau, err, B, compact=compact)
            assert_same(p, c, p_ref, c_ref, f"sweep {case} compact={compact}")
        p, c = dp.spdy_dp_solve_checkpointed(tau_d, err_d, B, int(rng.integers(0, 5)))
        torch.cuda.synchronize()
        assert_same(p.cpu().numpy(), c.cpu().numpy(), p_ref, c_ref, f"sweep {case} checkpointed")
        budgets = [B, B // 2, max(0, B - 1)]
        p, c = dp.spdy_dp_solve_budgets(tau_d, err_d, budgets)
        torch.cuda.synchronize()
        pb, cb = oracle.solve_budgets_ref(tau, err, budgets)
        for j in range(len(budgets)):
            assert_same(p[j].cpu().numpy(), c[j].cpu().numpy(), pb[j], cb[j],
                        f"sweep {case} budget {budgets[j]}")
        cs = rng.random((K, L)).astype(np.float32)
        w = np.sort(rng.random(S)).astype(np.float32)
        p, c = dp.spdy_dp_solve_sensitivities(tau_d, torch.from_numpy(cs).to(dev),
                                              torch.from_numpy(w).to(dev), B)
        torch.cuda.synchronize()
        ps, cs_ref = oracle.solve_sens_ref(tau, cs, w, B)
        assert_same(p.cpu().numpy(), c.cpu().numpy(), ps, cs_ref, f"sweep {case} sensitivities")


def test_a_solve_captured_in_a_graph_replays_correctly(dp):
    """The library neither allocates nor synchronises, so a solve can be captured into a HIP
    graph; every replay, with eager work and synchronisations in between, must equal the oracle."""
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(606)
    K, L, S, B = 6, 9, 12, 2000
    tau, err, _ = workloads.random_instance(rng, K, L, S, B, tau_max=B // 4, integer_err=3)
    other = workloads.random_instance(rng, K, L, S, B, tau_max=B // 4)[1]
    p_ref, c_ref = oracle.solve_ref(tau, err, B)
    p_other, c_other = oracle.solve_ref(tau, other, B)
    tau_d = torch.from_numpy(tau).to(dev)
    err_d = torch.from_numpy(err).to(dev)        # the graph reads whatever this buffer holds
    ws = dp.alloc_workspace(K, L, S, B, dev)
    profile = torch.empty((K, L), dtype=torch.int16, device=dev)
    cost = torch.empty((K,), dtype=torch.float32, device=dev)
    dp.spdy_dp_solve_batched(tau_d, err_d, B, profile, cost, ws)     # warm up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            dp.spdy_dp_solve_batched(tau_d, err_d, B, profile, cost, ws)
    torch.cuda.synchronize()
    for rep in range(4):
        table, want = (err, (p_ref, c_ref)) if rep % 2 == 0 else (other, (p_other, c_other))
        err_d.copy_(torch.from_numpy(table).to(dev))
        profile.fill_(-9)
        cost.fill_(-9.0)
        eager_p, eager_c = dp.spdy_dp_solve_batched(tau_d, err_d, B)  # eager work in between
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert_same(profile.cpu().numpy(), cost.cpu().numpy(), *want, f"replay {rep}")
        assert_same(eager_p.cpu().numpy(), eager_c.cpu().numpy(), *want, f"eager {rep}")


@pytest.mark.parametrize("compact, launch", [(False, 3), (True, 2)],
                         ids=["d_record_wide_in_place", "level_record_two_rows"])
def test_a_solve_that_needs_the_larger_lds_launch_replays_from_a_graph(dp, compact, launch):
    """Rows too long for the usual in-place launch take a launch with a larger LDS allocation
    (D record: the wide in-place one; level record: two alternating rows), whose attribute is
    set by the call itself; that call, captured, must replay correctly too."""
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(607)
    K, L, S, B = 3, 6, 10, 17000
    tau, err, _ = workloads.random_instance(rng, K, L, S, B, tau_max=B // 3, integer_err=3)
    other = workloads.random_instance(rng, K, L, S, B, tau_max=B // 3)[1]
    p_ref, c_ref = oracle.solve_ref(tau, err, B)
    p_other, c_other = oracle.solve_ref(tau, other, B)
    tau_d = torch.from_numpy(tau).to(dev)
    err_d = torch.from_numpy(err).to(dev)
    ws = dp.alloc_workspace(K, L, S, B, dev, compact=compact)
    profile = torch.empty((K, L), dtype=torch.int16, device=dev)
    cost = torch.empty((K,), dtype=torch.float32, device=dev)
    dp.spdy_dp_solve_batched(tau_d, err_d, B, profile, cost, ws)
    torch.cuda.synchronize()
    lay = dp.spdy_dp_workspace_layout(K, L, S, B, ws.numel())
    path = int(ws[lay["meta_offset"] + 12:lay["meta_offset"] + 16].cpu().numpy().view(np.int32)[0])
    assert path == launch, "this shape is meant to take the launch with the larger allocation"
    assert_same(profile.cpu().numpy(), cost.cpu().numpy(), p_ref, c_ref, "eager")
    graph = torch.cuda.CUDAGraph()
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            dp.spdy_dp_solve_batched(tau_d, err_d, B, profile, cost, ws)
    torch.cuda.synchronize()
    for rep in range(4):
        table, want = (err, (p_ref, c_ref)) if rep % 2 == 0 else (other, (p_other, c_other))
        err_d.copy_(torch.from_numpy(table).to(dev))
        profile.fill_(-9)
        cost.fill_(-9.0)
        eager_p, eager_c = dp.spdy_dp_solve_batched(tau_d, err_d, B)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert_same(profile.cpu().numpy(), cost.cpu().numpy(), *want, f"replay {rep}")
        assert_same(eager_p.cpu().numpy(), eager_c.cpu().numpy(), *want, f"eager {rep}")


def test_a_side_stream_with_the_wrappers_own_workspace(dp):
    """With no workspace given the wrapper allocates one and drops it on return, while the kernels
    are still queued on the caller's stream; allocations made right after on another stream must
    not get that block before the solve is done."""
    dev = torch.device("cuda:0")
    tau, err, B = workloads.generate(workloads.CONFIGS["rn50_k1"], K=24)
    p_ref, c_ref = oracle.solve_ref(tau, err, B, threads=CPU_THREADS)
    tau_d, err_d = torch.from_numpy(tau).to(dev), torch.from_numpy(err).to(dev)
    K, L, S = err.shape
    n = dp.spdy_dp_workspace_bytes(K, L, S, B)
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    for rep in range(3):
        side.wait_stream(torch.cuda.current_stream())
        profile, cost = dp.spdy_dp_solve_batched(tau_d, err_d, B, stream=side)
        # same-sized blocks on the current stream, scribbled over at once
        junk = [torch.empty(n, dtype=torch.uint8, device=dev).fill_(0x77) for _ in range(2)]
        side.synchronize()
        torch.cuda.synchronize()
        assert_same(profile.cpu().numpy(), cost.cpu().numpy(), p_ref, c_ref, f"rep {rep}")
        del junk


def test_two_host_threads_on_their_own_streams(dp):
    """The library keeps no state between calls: two host threads, each with its own stream,
    workspace and problem shape, solve concurrently."""
    import threading
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(314)
    problems = []
    for (K, L, S, B) in [(9, 10, 12, 3000), (5, 7, 70, 30000)]:   # small and large LDS limits
        tau, err, _ = workloads.random_instance(rng, K, L, S, B, tau_max=B // 3, integer_err=4)
        problems.append((tau, err, B, oracle.solve_ref(tau, err, B)))
    failures = []

    def work(i):
        try:
            torch.cuda.set_device(dev)
            tau, err, B, (p_ref, c_ref) = problems[i]
            stream = torch.cuda.Stream()
            tau_d, err_d = torch.from_numpy(tau).to(dev), torch.from_numpy(err).to(dev)
            K, L, S = err.shape
            ws = dp.alloc_workspace(K, L, S, B, dev)
            torch.cuda.synchronize()
            for _ in range(15):
                profile, cost = dp.spdy_dp_solve_batched(tau_d, err_d, B, workspace=ws,
                                                         stream=stream)
                stream.synchronize()
                assert_same(profile.cpu().numpy(), cost.cpu().numpy(), p_ref, c_ref, f"thread {i}")
        except Exception as e:                      # report from the main thread
            failures.append(repr(e))

    threads = [threading.Thread(target=work, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not failures, failures


def test_one_workspace_reused_across_different_problems(dp):
    """Nothing a call leaves in the workspace may matter to the next one, whatever its shape."""
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(77)
    shapes = [(5, 9, 12, 1000), (3, 4, 70, 900), (40, 3, 5, 200), (2, 12, 33, 2500), (6, 2, 3, 50),
              (3, 9, 12, 1000)]
    big = max(dp.spdy_dp_workspace_bytes(*sh) for sh in shapes)
    ws = torch.empty(big, dtype=torch.uint8, device=dev)
    ws.fill_(0x5A)
    for i, (K, L, S, B) in enumerate(shapes):
        tau, err, _ = workloads.random_instance(rng, K, L, S, B, tau_max=max(1, B // L),
                                                integer_err=3 if i % 2 else None,
                                                zero_tau_frac=0.1)
        p_ref, c_ref = oracle.solve_ref(tau, err, B)
        for nbytes in (big, dp.spdy_dp_workspace_bytes_min(K, L, S, B)):   # D record, level record
            profile, cost = dp.spdy_dp_solve_batched(torch.from_numpy(tau).to(dev),
                                                     torch.from_numpy(err).to(dev), B,
                                                     workspace=ws[:nbytes])
            torch.cuda.synchronize()
            assert_same(profile.cpu().numpy(), cost.cpu().numpy(), p_ref, c_ref,
                        f"problem {i} {(K, L, S, B)} bytes {nbytes}")


def test_workspace_too_small_is_an_error(dp):
    dev = torch.device("cuda:0")
    tau = torch.ones((2, 2), dtype=torch.int32, device=dev)
    err = torch.zeros((1, 2, 2), dtype=torch.float32, device=dev)
    ws = torch.empty(16, dtype=torch.uint8, device=dev)
    with pytest.raises(dp.SpdyDpError) as e:
        dp.spdy_dp_solve_batched(tau, err, 100, workspace=ws)
    assert e.value.status == -4
