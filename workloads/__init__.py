"""Seeded synthetic inputs (no SpMM arithmetic lives here)."""
from .generators import (CSR, CONFIGS, csr_from_sorted_keys, dense_B, from_coo, hidden_communities,
                         make_config, pruned_weight, rmat_gcn, stencil27, uniform_rows)

__all__ = ["CSR", "CONFIGS", "csr_from_sorted_keys", "dense_B", "from_coo", "hidden_communities",
           "make_config", "pruned_weight", "rmat_gcn", "stencil27", "uniform_rows"]
