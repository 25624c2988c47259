"""MI355X-native batched solver for the constrained layer-wise compression dynamic program
(Sec. 3.2, App. A Alg. 1).  The computation lives in ``csrc/spdy_dp.hip`` behind the C ABI
declared in ``include/spdy_dp.h``; ``binding`` marshals arguments to it."""
from .binding import (SpdyDpError, alloc_workspace, spdy_dp_backtrace, spdy_dp_fill,
                      spdy_dp_solve_batched, spdy_dp_solve_batched_static,
                      spdy_dp_solve_budgets, spdy_dp_solve_checkpointed,
                      spdy_dp_solve_from_incumbent, spdy_dp_solve_sensitivities, spdy_dp_strerror,
                      spdy_dp_workspace_bytes, spdy_dp_workspace_bytes_checkpointed,
                      spdy_dp_workspace_bytes_min, spdy_dp_workspace_layout)

__all__ = ["SpdyDpError", "alloc_workspace", "spdy_dp_backtrace", "spdy_dp_fill",
           "spdy_dp_solve_batched", "spdy_dp_solve_batched_static", "spdy_dp_solve_budgets",
           "spdy_dp_solve_checkpointed",
           "spdy_dp_solve_from_incumbent", "spdy_dp_solve_sensitivities", "spdy_dp_strerror",
           "spdy_dp_workspace_bytes", "spdy_dp_workspace_bytes_checkpointed",
           "spdy_dp_workspace_bytes_min", "spdy_dp_workspace_layout"]
