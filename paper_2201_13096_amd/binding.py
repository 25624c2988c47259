"""ctypes binding of ``libspdy_dp.so`` (declared in ``include/spdy_dp.h``).

Marshalling only: every step of Alg. 1 runs in the HIP kernels.  PyTorch supplies device memory
and the stream.  There is no CPU fallback: a missing library or a non-GPU tensor is an error.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspdy_dp.so")
_lib = None

OK = 0
ERR_NULL, ERR_DIM, ERR_LEVELS, ERR_WORKSPACE, ERR_OVERFLOW, ERR_LAUNCH = -1, -2, -3, -4, -5, -9
ERR_STATIC_LIMIT = -10
STATIC_WORKSPACE_BYTES = 64 << 20     # SPDY_DP_STATIC_WORKSPACE_BYTES in the header

EXPORTS = ("spdy_dp_workspace_bytes", "spdy_dp_workspace_bytes_min", "spdy_dp_solve_batched",
           "spdy_dp_solve_batched_static",
           "spdy_dp_solve_sensitivities", "spdy_dp_solve_budgets",
           "spdy_dp_solve_from_incumbent", "spdy_dp_workspace_bytes_checkpointed",
           "spdy_dp_solve_checkpointed", "spdy_dp_fill", "spdy_dp_backtrace",
           "spdy_dp_workspace_layout", "spdy_dp_strerror")


class SpdyDpError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"spdy_dp status {status}: {spdy_dp_strerror(status)}")


def lib() -> ctypes.CDLL:
    """Load the HIP library built in-tree; fails loudly if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it first (python -m paper_2201_13096_amd.build); "
                "there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        L.spdy_dp_workspace_bytes.restype = sz
        L.spdy_dp_workspace_bytes.argtypes = [i, i, i, i]
        L.spdy_dp_workspace_bytes_min.restype = sz
        L.spdy_dp_workspace_bytes_min.argtypes = [i, i, i, i]
        L.spdy_dp_solve_batched.restype = i
        L.spdy_dp_solve_batched.argtypes = [vp, vp, i, i, i, i, vp, vp, vp, sz, vp]
        L.spdy_dp_solve_batched_static.restype = i
        L.spdy_dp_solve_batched_static.argtypes = [vp, vp, i, i, i, i, vp, vp, vp]
        L.spdy_dp_solve_sensitivities.restype = i
        L.spdy_dp_solve_sensitivities.argtypes = [vp, vp, vp, i, i, i, i, vp, vp, vp, sz, vp]
        L.spdy_dp_solve_budgets.restype = i
        L.spdy_dp_solve_budgets.argtypes = [vp, vp, i, i, i, ctypes.POINTER(ctypes.c_int32), i, vp,
                                            vp, vp, sz, vp]
        L.spdy_dp_solve_from_incumbent.restype = i
        L.spdy_dp_solve_from_incumbent.argtypes = [vp, vp, vp, i, i, i, i, vp, sz, vp, vp, vp, sz,
                                                   vp]
        L.spdy_dp_workspace_bytes_checkpointed.restype = sz
        L.spdy_dp_workspace_bytes_checkpointed.argtypes = [i, i, i, i, i]
        L.spdy_dp_solve_checkpointed.restype = i
        L.spdy_dp_solve_checkpointed.argtypes = [vp, vp, i, i, i, i, i, vp, vp, vp, sz, vp]
        L.spdy_dp_fill.restype = i
        L.spdy_dp_fill.argtypes = [vp, vp, i, i, i, i, vp, vp, sz, vp]
        L.spdy_dp_backtrace.restype = i
        L.spdy_dp_backtrace.argtypes = [vp, vp, i, i, i, i, vp, vp, vp, sz, vp]
        L.spdy_dp_workspace_layout.restype = i
        L.spdy_dp_workspace_layout.argtypes = [i, i, i, i, sz, ctypes.POINTER(sz)]
        L.spdy_dp_strerror.restype = ctypes.c_char_p
        L.spdy_dp_strerror.argtypes = [i]
        _lib = L
    return _lib


def spdy_dp_strerror(status: int) -> str:
    return lib().spdy_dp_strerror(int(status)).decode()


def spdy_dp_workspace_bytes(K: int, L: int, S: int, B: int) -> int:
    return int(lib().spdy_dp_workspace_bytes(K, L, S, B))


def spdy_dp_workspace_bytes_min(K: int, L: int, S: int, B: int) -> int:
    return int(lib().spdy_dp_workspace_bytes_min(K, L, S, B))


def spdy_dp_workspace_layout(K: int, L: int, S: int, B: int, workspace_bytes: int) -> dict:
    """Where things are in a workspace of that size (see the header): variant (0 = fp32 D
    record, 1 = one-byte level record), byte offsets, record pitch and rows per candidate."""
    out = (ctypes.c_size_t * 8)()
    st = lib().spdy_dp_workspace_layout(K, L, S, B, int(workspace_bytes), out)
    if st != OK:
        raise SpdyDpError(st)
    keys = ("variant", "meta_offset", "tstar_offset", "record_offset", "record_pitch",
            "record_rows", "header_words", "plan_words")
    return dict(zip(keys, (int(v) for v in out)))


def _dev(t: torch.Tensor, dtype, name: str) -> torch.Tensor:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a tensor on the GPU")
    if t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name} must be contiguous {dtype}")
    return t


def _shapes(tau: torch.Tensor, err: torch.Tensor):
    if tau.dim() != 2 or err.dim() != 3 or tuple(err.shape[1:]) != tuple(tau.shape):
        raise ValueError("tau must be [L, S] and err [K, L, S]")
    K, L, S = err.shape
    return int(K), int(L), int(S)


def _stream(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def alloc_workspace(K: int, L: int, S: int, B: int, device=None, compact: bool = False):
    """Workspace tensor: the fast fp32-record size, or the 4x smaller level-record size."""
    n = (spdy_dp_workspace_bytes_min if compact else spdy_dp_workspace_bytes)(K, L, S, B)
    if n == 0:
        raise _size_error(K, L, S, B)
    return torch.empty(n, dtype=torch.uint8, device=device or "cuda")


def _size_error(K: int, L: int, S: int, B: int) -> "SpdyDpError":
    return SpdyDpError(lib().spdy_dp_workspace_layout(K, L, S, B, 2 ** 62,
                                                      (ctypes.c_size_t * 8)()))


def _own_workspace(n: int, device, stream):
    """A workspace the wrapper allocates itself and drops when it returns, while the kernels that
    use it are still queued on ``stream``: the caching allocator is told about that stream, so
    it does not hand the block to other work before those kernels are done."""
    ws = torch.empty(n, dtype=torch.uint8, device=device)
    if stream is not None:
        ws.record_stream(stream)
    return ws


def _own_full_workspace(K: int, L: int, S: int, B: int, device, stream):
    n = spdy_dp_workspace_bytes(K, L, S, B)
    if n == 0:
        raise _size_error(K, L, S, B)
    return _own_workspace(n, device, stream)


def spdy_dp_solve_batched(tau, err, B: int, profile=None, cost=None, workspace=None, stream=None):
    """Whole of Alg. 1 for K candidates.  Returns ``(profile int16[K,L], cost fp32[K])`` (device
    tensors, valid after the stream is synchronised)."""
    tau = _dev(tau, torch.int32, "tau")
    err = _dev(err, torch.float32, "err")
    K, L, S = _shapes(tau, err)
    if profile is None:
        profile = torch.empty((K, L), dtype=torch.int16, device=err.device)
    if cost is None:
        cost = torch.empty((K,), dtype=torch.float32, device=err.device)
    if workspace is None:
        workspace = _own_full_workspace(K, L, S, B, err.device, stream)
    _dev(profile, torch.int16, "profile")
    _dev(cost, torch.float32, "cost")
    _dev(workspace, torch.uint8, "workspace")
    st = lib().spdy_dp_solve_batched(tau.data_ptr(), err.data_ptr(), K, L, S, int(B),
                                     profile.data_ptr(), cost.data_ptr(), workspace.data_ptr(),
                                     workspace.numel(), _stream(stream))
    if st != OK:
        raise SpdyDpError(st)
    return profile, cost


def spdy_dp_solve_batched_static(tau, err, B: int, profile=None, cost=None, stream=None):
    """``spdy_dp_solve_batched`` on the workspace built into the library (no allocation inside the
    call when ``profile`` and ``cost`` are given).  Calls that overlap on one GPU race."""
    tau = _dev(tau, torch.int32, "tau")
    err = _dev(err, torch.float32, "err")
    K, L, S = _shapes(tau, err)
    if profile is None:
        profile = torch.empty((K, L), dtype=torch.int16, device=err.device)
    if cost is None:
        cost = torch.empty((K,), dtype=torch.float32, device=err.device)
    _dev(profile, torch.int16, "profile")
    _dev(cost, torch.float32, "cost")
    st = lib().spdy_dp_solve_batched_static(tau.data_ptr(), err.data_ptr(), K, L, S, int(B),
                                            profile.data_ptr(), cost.data_ptr(), _stream(stream))
    if st != OK:
        raise SpdyDpError(st)
    return profile, cost


def spdy_dp_solve_sensitivities(tau, c, w, B: int, profile=None, cost=None, workspace=None,
                                stream=None):
    """Alg. 1 for err[k,l,s] = c[k,l] * w[s] (Eq. 4) without materialising the table."""
    tau = _dev(tau, torch.int32, "tau")
    c = _dev(c, torch.float32, "c")
    w = _dev(w, torch.float32, "w")
    if tau.dim() != 2 or c.dim() != 2 or w.dim() != 1 or c.shape[1] != tau.shape[0] \
            or w.shape[0] != tau.shape[1]:
        raise ValueError("tau must be [L, S], c [K, L] and w [S]")
    K, L, S = int(c.shape[0]), int(tau.shape[0]), int(tau.shape[1])
    if profile is None:
        profile = torch.empty((K, L), dtype=torch.int16, device=c.device)
    if cost is None:
        cost = torch.empty((K,), dtype=torch.float32, device=c.device)
    if workspace is None:
        workspace = _own_full_workspace(K, L, S, B, c.device, stream)
    _dev(profile, torch.int16, "profile")
    _dev(cost, torch.float32, "cost")
    _dev(workspace, torch.uint8, "workspace")
    st = lib().spdy_dp_solve_sensitivities(tau.data_ptr(), c.data_ptr(), w.data_ptr(), K, L, S,
                                           int(B), profile.data_ptr(), cost.data_ptr(),
                                           workspace.data_ptr(), workspace.numel(),
                                           _stream(stream))
    if st != OK:
        raise SpdyDpError(st)
    return profile, cost


def spdy_dp_solve_budgets(tau, err, budgets, profile=None, cost=None, workspace=None,
                          stream=None):
    """One fill for max(budgets), then argmin and walk back per budget.  Returns
    ``(profile int16[J,K,L], cost fp32[J,K])``."""
    tau = _dev(tau, torch.int32, "tau")
    err = _dev(err, torch.float32, "err")
    K, L, S = _shapes(tau, err)
    budgets = [int(b) for b in budgets]
    J = len(budgets)
    if J == 0:
        raise ValueError("at least one budget")
    arr = (ctypes.c_int32 * J)(*budgets)
    if profile is None:
        profile = torch.empty((J, K, L), dtype=torch.int16, device=err.device)
    if cost is None:
        cost = torch.empty((J, K), dtype=torch.float32, device=err.device)
    if workspace is None:
        workspace = _own_full_workspace(K, L, S, max(budgets), err.device, stream)
    _dev(profile, torch.int16, "profile")
    _dev(cost, torch.float32, "cost")
    _dev(workspace, torch.uint8, "workspace")
    st = lib().spdy_dp_solve_budgets(tau.data_ptr(), err.data_ptr(), K, L, S, arr, J,
                                     profile.data_ptr(), cost.data_ptr(), workspace.data_ptr(),
                                     workspace.numel(), _stream(stream))
    if st != OK:
        raise SpdyDpError(st)
    return profile, cost


def spdy_dp_solve_from_incumbent(tau, err, first_layer, B: int, incumbent_workspace,
                                 profile=None, cost=None, workspace=None, stream=None):
    """Re-solve candidates whose tables equal a solved incumbent's before ``first_layer[k]``."""
    tau = _dev(tau, torch.int32, "tau")
    err = _dev(err, torch.float32, "err")
    first_layer = _dev(first_layer, torch.int32, "first_layer")
    _dev(incumbent_workspace, torch.uint8, "incumbent_workspace")
    K, L, S = _shapes(tau, err)
    if first_layer.numel() != K:
        raise ValueError("first_layer must have K entries")
    if profile is None:
        profile = torch.empty((K, L), dtype=torch.int16, device=err.device)
    if cost is None:
        cost = torch.empty((K,), dtype=torch.float32, device=err.device)
    if workspace is None:
        workspace = _own_full_workspace(K, L, S, B, err.device, stream)
    _dev(profile, torch.int16, "profile")
    _dev(cost, torch.float32, "cost")
    _dev(workspace, torch.uint8, "workspace")
    st = lib().spdy_dp_solve_from_incumbent(
        tau.data_ptr(), err.data_ptr(), first_layer.data_ptr(), K, L, S, int(B),
        incumbent_workspace.data_ptr(), incumbent_workspace.numel(), profile.data_ptr(),
        cost.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream(stream))
    if st != OK:
        raise SpdyDpError(st)
    return profile, cost


def spdy_dp_workspace_bytes_checkpointed(K: int, L: int, S: int, B: int, stride: int = 0) -> int:
    return int(lib().spdy_dp_workspace_bytes_checkpointed(K, L, S, B, stride))


def spdy_dp_solve_checkpointed(tau, err, B: int, stride: int = 0, profile=None, cost=None,
                               workspace=None, stream=None):
    """Alg. 1 with about 2 sqrt(L) rows of record per candidate (two fills)."""
    tau = _dev(tau, torch.int32, "tau")
    err = _dev(err, torch.float32, "err")
    K, L, S = _shapes(tau, err)
    if profile is None:
        profile = torch.empty((K, L), dtype=torch.int16, device=err.device)
    if cost is None:
        cost = torch.empty((K,), dtype=torch.float32, device=err.device)
    if workspace is None:
        n = spdy_dp_workspace_bytes_checkpointed(K, L, S, B, stride)
        if n == 0:
            raise SpdyDpError(lib().spdy_dp_solve_checkpointed(None, None, K, L, S, int(B), stride,
                                                               None, None, None, 0, None))
        workspace = _own_workspace(n, err.device, stream)
    _dev(profile, torch.int16, "profile")
    _dev(cost, torch.float32, "cost")
    _dev(workspace, torch.uint8, "workspace")
    st = lib().spdy_dp_solve_checkpointed(tau.data_ptr(), err.data_ptr(), K, L, S, int(B),
                                          int(stride), profile.data_ptr(), cost.data_ptr(),
                                          workspace.data_ptr(), workspace.numel(), _stream(stream))
    if st != OK:
        raise SpdyDpError(st)
    return profile, cost


def spdy_dp_fill(tau, err, B: int, cost, workspace, stream=None) -> None:
    tau = _dev(tau, torch.int32, "tau")
    err = _dev(err, torch.float32, "err")
    K, L, S = _shapes(tau, err)
    _dev(cost, torch.float32, "cost")
    _dev(workspace, torch.uint8, "workspace")
    st = lib().spdy_dp_fill(tau.data_ptr(), err.data_ptr(), K, L, S, int(B), cost.data_ptr(),
                            workspace.data_ptr(), workspace.numel(), _stream(stream))
    if st != OK:
        raise SpdyDpError(st)


def spdy_dp_backtrace(tau, err, B: int, profile, cost, workspace, stream=None) -> None:
    tau = _dev(tau, torch.int32, "tau")
    err = _dev(err, torch.float32, "err")
    K, L, S = _shapes(tau, err)
    _dev(profile, torch.int16, "profile")
    _dev(cost, torch.float32, "cost")
    _dev(workspace, torch.uint8, "workspace")
    st = lib().spdy_dp_backtrace(tau.data_ptr(), err.data_ptr(), K, L, S, int(B),
                                 profile.data_ptr(), cost.data_ptr(), workspace.data_ptr(),
                                 workspace.numel(), _stream(stream))
    if st != OK:
        raise SpdyDpError(st)
