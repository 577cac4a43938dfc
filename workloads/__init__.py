"""Seeded synthetic inputs shaped like the paper's workloads.

The paper measures MTTKRP and TTMc on FROSTT tensors (Sec. 5.2, 5.3, Table 2)
and introduces the three-tensor product Z_im = U_ijk V_jl W_klm (Sec. 1).  None
of those data sets is used here: the generators below make stand-ins with the
same order, extents, nonzero counts and power-law skew.  They serve both the
CPU oracle and the GPU library and contain none of the method's arithmetic.
"""
from .generators import (SparseCOO, Workload, zipf_cdf, distinct_coords,
                         block_sparse_coords, dense_factor, sparse_values,
                         make_ttmc3, make_ttmc4, make_mttkrp3, make_sptn3)
from .configs import CONFIGS, SMALL, make, BASE_SEED

__all__ = ["SparseCOO", "Workload", "zipf_cdf", "distinct_coords",
           "block_sparse_coords", "dense_factor", "sparse_values",
           "make_ttmc3", "make_ttmc4", "make_mttkrp3", "make_sptn3",
           "CONFIGS", "SMALL", "make", "BASE_SEED"]
