"""MI355X-native hot path of HessFormer's stochastic Lanczos quadrature:
Hessian-vector products of language-model losses and the Lanczos iteration
around them, as hand-written HIP kernels behind a C ABI (include/hessformer.h).
This package is the thin ctypes binding of that library."""
from .binding import (Context, HessformerError, hf_desc_num_params, hf_layout, hf_tridiag_readout, hf_version,
                      hf_slq_density, hf_slq_moments, hf_column_stats_noalloc, make_desc, lib, EXPORTS, LIB_PATH)

__all__ = ["Context", "HessformerError", "hf_desc_num_params", "hf_layout", "hf_tridiag_readout", "hf_version",
           "hf_slq_density", "hf_slq_moments", "hf_column_stats_noalloc", "make_desc", "lib", "EXPORTS", "LIB_PATH"]
