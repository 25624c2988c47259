"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every function the
header declares, sizes its workspace as documented and rejects bad arguments before touching
the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "spdy_dp.h")


@pytest.fixture(scope="module")
def binding():
    from paper_2201_13096_amd import binding as b
    if not os.path.exists(b.LIB_PATH):
        from paper_2201_13096_amd import build
        build.build_library()
    return b


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spdy_dp_\w+)\s*\(", text)))


def test_library_exports_every_declared_function(binding):
    names = declared_functions()
    assert len(names) >= 9
    lib = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def test_status_codes_match_header(binding):
    text = open(HEADER).read()
    codes = dict(re.findall(r"#define\s+SPDY_DP_(\w+)\s+\(?(-?\d+)\)?", text))
    assert int(codes["OK"]) == binding.OK
    assert int(codes["ERR_NULL"]) == binding.ERR_NULL
    assert int(codes["ERR_DIM"]) == binding.ERR_DIM
    assert int(codes["ERR_LEVELS"]) == binding.ERR_LEVELS
    assert int(codes["ERR_WORKSPACE"]) == binding.ERR_WORKSPACE
    assert int(codes["ERR_OVERFLOW"]) == binding.ERR_OVERFLOW
    assert int(codes["ERR_LAUNCH"]) == binding.ERR_LAUNCH
    for v in codes.values():
        assert binding.spdy_dp_strerror(int(v)) != "unknown status"
    assert binding.spdy_dp_strerror(-1234) == "unknown status"


def test_workspace_size(binding):
    K, L, S, B = 1024, 54, 40, 10000
    row = (B + 1 + 63) // 64 * 64
    fast = binding.spdy_dp_workspace_bytes(K, L, S, B)
    small = binding.spdy_dp_workspace_bytes_min(K, L, S, B)
    # fp32 D per cell (one extra row per candidate) vs one byte per cell, rows padded to 64
    # per (layer, level): shifts, visiting order, entry starts (8 more per layer), entry of a level
    tables = 4 * 4 * L * ((S + 7) // 8 * 8) + 4 * 8 * L
    assert 4 * K * L * row + tables <= fast <= 4 * K * L * row + tables + 16384
    assert K * L * row + tables <= small <= K * L * row + tables + 16384
    lay = binding.spdy_dp_workspace_layout(K, L, S, B, fast)
    assert lay["variant"] == 0 and lay["record_pitch"] == row and lay["record_rows"] == L
    lay = binding.spdy_dp_workspace_layout(K, L, S, B, fast - 1)
    assert lay["variant"] == 1 and lay["record_pitch"] == row and lay["record_rows"] == L
    assert lay["record_offset"] % 256 == 0 and lay["tstar_offset"] % 256 == 0
    assert lay["tstar_offset"] >= 4 * (8 + 2 * L) + tables
    assert lay["record_offset"] >= lay["tstar_offset"] + 4 * K
    with pytest.raises(binding.SpdyDpError) as e:
        binding.spdy_dp_workspace_layout(K, L, S, B, small - 1)
    assert e.value.status == binding.ERR_WORKSPACE
    # rows that may not fit LDS add two fp32 rows per candidate
    K, L, S, B = 256, 200, 64, 65536
    row = (B + 1 + 63) // 64 * 64
    assert binding.spdy_dp_workspace_bytes_min(K, L, S, B) >= K * L * row + 2 * K * row * 4
    assert binding.spdy_dp_workspace_bytes(K, L, S, B) >= 4 * K * L * row + 2 * K * row * 4
    # the record with checkpoints: L / stride - 1 checkpoint rows + stride block rows per candidate
    K, L, S, B = 256, 200, 64, 65536
    row = (B + 1 + 63) // 64 * 64
    full = binding.spdy_dp_workspace_bytes(K, L, S, B)
    auto = binding.spdy_dp_workspace_bytes_checkpointed(K, L, S, B, 0)      # stride 15
    spill = 2 * K * (row + 1792) * 4            # two rows per candidate in memory (long rows)
    assert 4 * K * (13 + 15) * row + spill <= auto <= 4 * K * (13 + 15) * row + spill + (1 << 20)
    assert auto * 5 < full
    assert binding.spdy_dp_workspace_bytes_checkpointed(K, L, S, B, 10) == \
        binding.spdy_dp_workspace_bytes_checkpointed(K, L, S, B, 20)        # 19 + 10 = 9 + 20
    assert binding.spdy_dp_workspace_bytes_checkpointed(K, L, S, B, 1000) >= full   # one block
    assert binding.spdy_dp_workspace_bytes_checkpointed(K, 0, S, B, 0) == 0
    # invalid sizes -> 0
    for f in (binding.spdy_dp_workspace_bytes, binding.spdy_dp_workspace_bytes_min):
        assert f(0, 1, 1, 1) == 0
        assert f(1, 1, 1, -1) == 0
        assert f(1, 1, 256, 1) == 0
        assert f(1, 1, 255, 1) > 0
        assert f(2 ** 31 - 1, 2 ** 31 - 1, 255, 2 ** 31 - 2000) == 0


def test_argument_errors_are_reported_before_any_launch(binding):
    lib = binding.lib()
    fake = 0x1000  # never dereferenced: every call below must fail validation first
    solve = lib.spdy_dp_solve_batched
    assert solve(None, fake, 1, 1, 1, 1, fake, fake, fake, 1 << 20, None) == binding.ERR_NULL
    assert solve(fake, None, 1, 1, 1, 1, fake, fake, fake, 1 << 20, None) == binding.ERR_NULL
    assert solve(fake, fake, 1, 1, 1, 1, None, fake, fake, 1 << 20, None) == binding.ERR_NULL
    assert solve(fake, fake, 1, 1, 1, 1, fake, None, fake, 1 << 20, None) == binding.ERR_NULL
    assert solve(fake, fake, 1, 1, 1, 1, fake, fake, None, 1 << 20, None) == binding.ERR_NULL
    assert solve(fake, fake, 0, 1, 1, 1, fake, fake, fake, 1 << 20, None) == binding.ERR_DIM
    assert solve(fake, fake, 1, 0, 1, 1, fake, fake, fake, 1 << 20, None) == binding.ERR_DIM
    assert solve(fake, fake, 1, 1, 0, 1, fake, fake, fake, 1 << 20, None) == binding.ERR_DIM
    assert solve(fake, fake, 1, 1, 1, -1, fake, fake, fake, 1 << 20, None) == binding.ERR_DIM
    assert solve(fake, fake, 1, 1, 256, 1, fake, fake, fake, 1 << 20, None) == binding.ERR_LEVELS
    assert solve(fake, fake, 1, 1, 1, 1, fake, fake, fake, 8, None) == binding.ERR_WORKSPACE
    assert solve(fake, fake, 2 ** 31 - 1, 2 ** 31 - 1, 2, 2 ** 31 - 2000, fake, fake, fake,
                 1 << 20, None) == binding.ERR_OVERFLOW
    one = (ctypes.c_int32 * 2)(5, 9)
    neg = (ctypes.c_int32 * 2)(5, -1)
    multi = lib.spdy_dp_solve_budgets
    assert multi(fake, fake, 1, 1, 1, None, 2, fake, fake, fake, 1 << 20, None) == binding.ERR_NULL
    assert multi(fake, fake, 1, 1, 1, one, 0, fake, fake, fake, 1 << 20, None) == binding.ERR_DIM
    assert multi(fake, fake, 1, 1, 1, neg, 2, fake, fake, fake, 1 << 20, None) == binding.ERR_DIM
    assert multi(fake, fake, 1, 1, 1, one, 2, fake, fake, fake, 8, None) == binding.ERR_WORKSPACE
    sens = lib.spdy_dp_solve_sensitivities
    assert sens(fake, None, fake, 1, 1, 1, 1, fake, fake, fake, 1 << 20, None) == binding.ERR_NULL
    assert sens(fake, fake, None, 1, 1, 1, 1, fake, fake, fake, 1 << 20, None) == binding.ERR_NULL
    assert sens(fake, fake, fake, 1, 1, 300, 1, fake, fake, fake, 1 << 20, None) == \
        binding.ERR_LEVELS
    inc = lib.spdy_dp_solve_from_incumbent
    big = 1 << 20
    far = 0x40000000
    assert inc(fake, fake, None, 1, 1, 1, 1, far, big, fake, fake, fake, big, None) == \
        binding.ERR_NULL
    assert inc(fake, None, fake, 1, 1, 1, 1, far, big, fake, fake, fake, big, None) == \
        binding.ERR_NULL
    assert inc(fake, fake, fake, 1, 1, 1, 1, None, big, fake, fake, fake, big, None) == \
        binding.ERR_NULL
    assert inc(fake, fake, fake, 1, 0, 1, 1, far, big, fake, fake, fake, big, None) == \
        binding.ERR_DIM
    assert inc(fake, fake, fake, 1, 1, 1, 1, far, 8, fake, fake, fake, big, None) == \
        binding.ERR_WORKSPACE
    assert inc(fake, fake, fake, 1, 1, 1, 1, far, big, fake, fake, fake, 8, None) == \
        binding.ERR_WORKSPACE
    # overlapping workspaces: the fill would overwrite the rows it resumes from
    assert inc(fake, fake, fake, 1, 1, 1, 1, fake + 64, big, fake, fake, fake, big, None) == \
        binding.ERR_WORKSPACE
    # a level-record workspace keeps no rows of D to resume from
    small = binding.lib().spdy_dp_workspace_bytes_min(4, 8, 8, 1000)
    assert small < binding.lib().spdy_dp_workspace_bytes(4, 8, 8, 1000)
    assert inc(fake, fake, fake, 4, 8, 8, 1000, far, big, fake, fake, fake, small, None) == \
        binding.ERR_WORKSPACE
    ck = lib.spdy_dp_solve_checkpointed
    assert ck(fake, None, 1, 1, 1, 1, 0, fake, fake, fake, big, None) == binding.ERR_NULL
    assert ck(None, fake, 1, 1, 1, 1, 0, fake, fake, fake, big, None) == binding.ERR_NULL
    assert ck(fake, fake, 1, 1, 1, 1, 0, None, fake, fake, big, None) == binding.ERR_NULL
    assert ck(fake, fake, 1, 0, 1, 1, 0, fake, fake, fake, big, None) == binding.ERR_DIM
    assert ck(fake, fake, 1, 1, 300, 1, 0, fake, fake, fake, big, None) == binding.ERR_LEVELS
    assert ck(fake, fake, 1, 1, 1, 1, 0, fake, fake, fake, 8, None) == binding.ERR_WORKSPACE
    # the workspace of one stride does not serve a stride that needs more rows
    need4 = binding.spdy_dp_workspace_bytes_checkpointed(8, 64, 8, 4000, 4)
    need8 = binding.spdy_dp_workspace_bytes_checkpointed(8, 64, 8, 4000, 8)
    assert need8 < need4 < binding.spdy_dp_workspace_bytes(8, 64, 8, 4000)
    assert ck(fake, fake, 8, 64, 8, 4000, 4, fake, fake, fake, need8, None) == \
        binding.ERR_WORKSPACE
    assert lib.spdy_dp_fill(fake, fake, 1, 1, 1, 1, None, fake, 1 << 20, None) == binding.ERR_NULL
    bt = lib.spdy_dp_backtrace
    assert bt(fake, fake, 1, 1, 1, 1, None, fake, fake, 1 << 20, None) == binding.ERR_NULL
    assert bt(fake, None, 1, 1, 1, 1, fake, fake, fake, 1 << 20, None) == binding.ERR_NULL
    assert bt(fake, fake, 1, 1, 1, 1, fake, None, fake, 1 << 20, None) == binding.ERR_NULL
    assert bt(fake, fake, 1, 1, 1, 1, fake, fake, fake, 8, None) == binding.ERR_WORKSPACE


def test_binding_refuses_cpu_tensors(binding):
    import torch
    tau = torch.zeros((2, 2), dtype=torch.int32)
    err = torch.zeros((1, 2, 2), dtype=torch.float32)
    with pytest.raises(TypeError):
        binding.spdy_dp_solve_batched(tau, err, 4)
