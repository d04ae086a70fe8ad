"""Python binding of libnnrescal (non-negative RESCAL multiplicative updates with a fused perturbation
ensemble, hand-written HIP for gfx950).  The binding only marshals arguments: device memory and
streams come from PyTorch, every step of the method runs inside the shared library.  Function names
match the C ABI in include/nnrescal.h."""
from .binding import (DenseX, SparseX, load, lib_path, nnrescal_cluster, nnrescal_destroy, nnrescal_fit,  # noqa: F401
                      nnrescal_fit_until,
                      nnrescal_get_factors, nnrescal_init, nnrescal_last_error, nnrescal_mu_step,
                      nnrescal_objective, nnrescal_perturb, nnrescal_products, nnrescal_profile, nnrescal_select_k,
                      nnrescal_set_factors, nnrescal_start_nndsvd, nnrescal_mu_step_static, nnrescal_gather_form, NNRescalError, EXPORTED_SYMBOLS)
