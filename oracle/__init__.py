"""CPU oracle for non-negative RESCAL with a perturbation ensemble and model selection.

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain, fp64 reference that the HIP
library is checked against.  It shares no code with the HIP path, imports nothing from
`paper_2202_09512_amd`, and is imported only by `tests/`, `__graft_entry__.smoke()` and the
`cpu_baseline` leg of `bench.py`.  The product path never calls into it.

Modules (each function cites the passage of arxiv 2202.09512 it follows):
  philox   - Philox4x32-10 counter-based generator (Salmon et al., SC'11), two implementations
  perturb  - the resampling X^q = X (*) Delta^q (Alg. 4) and the random initialisation (Alg. 3 step 1)
  mu       - multiplicative updates (Eq. 2 / Alg. 3 with p = 1), normalisation, objective
  select   - custom clustering (Alg. 5), medians, silhouettes (Alg. 6), regression, error, k_opt (Alg. 1)
  nndsvd   - the SVD-based start (section "Experiments", algorithmic parameters, option 2)

Parity status: every function is pinned by `tests/test_oracle_*.py` except where a docstring says
"parity unpinned" (the choice of random stream, which the paper leaves open).
"""
