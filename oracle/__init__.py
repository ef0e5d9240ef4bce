"""CPU oracle of the blocked SpMM path -- TEST INFRASTRUCTURE.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package; the product (paper_2408_11551_amd) never does, and nothing here
imports the product.  See smat_ref.py for what is defined and from which part
of the paper.
"""
from .smat_ref import (  # noqa: F401
    decode16, spmm_ref, block_pattern, count_blocks, count_blocks_bruteforce,
    bcsr_from_csr, bcsr_from_csr_fast, cluster_from_seed, jaccard_reorder, choose_perm,
)
