"""The entry point that allocates nothing (``spdy_dp_solve_batched_static``: the workspace is an
array inside the library's code object) against ``spdy_dp_solve_batched`` with a caller-owned
workspace, through the C ABI: two calls in a row, the second on a smaller problem, bit for bit;
then a batch that only fits with the one-byte level record, and one that does not fit at all."""
import ctypes

import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def dp():
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2201_13096_amd as m
    m.binding.lib()
    return m


def solve_both(dp, tau, err, B):
    """Raw C-ABI calls of both entry points on the same device inputs."""
    lib = dp.binding.lib()
    dev = torch.device("cuda:0")
    K, L, S = err.shape
    tau_d = torch.from_numpy(tau).to(dev)
    err_d = torch.from_numpy(err).to(dev)
    ws = dp.alloc_workspace(K, L, S, B, dev)
    out = []
    for static in (False, True):
        profile = torch.full((K, L), -7, dtype=torch.int16, device=dev)
        cost = torch.full((K,), -7.0, dtype=torch.float32, device=dev)
        stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        if static:
            st = lib.spdy_dp_solve_batched_static(tau_d.data_ptr(), err_d.data_ptr(), K, L, S, B,
                                                  profile.data_ptr(), cost.data_ptr(), stream)
        else:
            st = lib.spdy_dp_solve_batched(tau_d.data_ptr(), err_d.data_ptr(), K, L, S, B,
                                           profile.data_ptr(), cost.data_ptr(), ws.data_ptr(),
                                           ws.numel(), stream)
        assert st == 0, dp.spdy_dp_strerror(st)
        torch.cuda.synchronize()
        out.append((profile.cpu().numpy(), cost.cpu().numpy(), free_before,
                    torch.cuda.mem_get_info()[0]))
    return out


def same_bits(a, b, what):
    assert (a[0] == b[0]).all(), f"{what}: profiles differ"
    assert (a[1].view(np.uint32) == b[1].view(np.uint32)).all(), f"{what}: cost bits differ"


def test_static_workspace_equals_caller_workspace_twice_in_a_row(dp):
    rng = np.random.default_rng(8)
    big = workloads.generate(workloads.CONFIGS["rn50_k1"], K=7)              # D record, 15 MB
    small = workloads.random_instance(rng, 3, 6, 9, 700, tau_max=200, integer_err=3,
                                      zero_tau_frac=0.1)                      # smaller, ties
    freed = []
    for name, (tau, err, B) in (("first", big), ("second, smaller", small), ("third", big)):
        print(f"[no-alloc] {name}: K={err.shape[0]} L={err.shape[1]} S={err.shape[2]} B={B}",
              flush=True)
        plain, static = solve_both(dp, tau, err, B)
        same_bits(static, plain, name)
        p_ref, c_ref = oracle.solve_ref(tau, err, B)
        same_bits(static, (p_ref, c_ref), name + " vs oracle")
        freed.append(static[3] - static[2])
    # device memory in use did not change across the later calls (the first one may load the
    # library's code object, which holds the array)
    assert freed[1] == 0 and freed[2] == 0, freed


def test_static_workspace_falls_back_to_the_level_record_and_reports_its_limit(dp):
    lib = dp.binding.lib()
    limit = dp.binding.STATIC_WORKSPACE_BYTES
    tau, err, B = workloads.generate(workloads.CONFIGS["rn50_k1"], K=40)
    K, L, S = err.shape
    assert dp.spdy_dp_workspace_bytes_min(K, L, S, B) <= limit < dp.spdy_dp_workspace_bytes(K, L, S, B)
    plain, static = solve_both(dp, tau, err, B)
    same_bits(static, plain, "level record")
    p_ref, c_ref = oracle.solve_ref(tau, err, B, threads=8)
    same_bits(static, (p_ref, c_ref), "level record vs oracle")
    # beyond the array: refused before anything is enqueued, outputs untouched
    dev = torch.device("cuda:0")
    K = 200
    assert dp.spdy_dp_workspace_bytes_min(K, L, S, B) > limit
    profile = torch.full((K, L), -7, dtype=torch.int16, device=dev)
    cost = torch.full((K,), -7.0, dtype=torch.float32, device=dev)
    tau_d = torch.from_numpy(tau).to(dev)
    err_d = torch.zeros((K, L, S), dtype=torch.float32, device=dev)
    st = lib.spdy_dp_solve_batched_static(tau_d.data_ptr(), err_d.data_ptr(), K, L, S, B,
                                          profile.data_ptr(), cost.data_ptr(), None)
    assert st == dp.binding.ERR_STATIC_LIMIT
    torch.cuda.synchronize()
    assert (profile == -7).all() and (cost == -7.0).all()
    with pytest.raises(dp.SpdyDpError) as e:
        dp.spdy_dp_solve_batched_static(tau_d, err_d, B)
    assert e.value.status == dp.binding.ERR_STATIC_LIMIT
