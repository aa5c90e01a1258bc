"""Row-structured hybrid SpMM for MI355X: Python binding of the C-ABI library."""
from .binding import (EXPORTED_SYMBOLS, Plan, RshError, lib, rsh_csr_t, rsh_plan_opts_default,
                      rsh_plan_opts_t, rsh_plan_stats_t)
from . import binding

__all__ = ["EXPORTED_SYMBOLS", "Plan", "RshError", "lib", "binding", "rsh_csr_t", "rsh_plan_opts_default",
           "rsh_plan_opts_t", "rsh_plan_stats_t"]
