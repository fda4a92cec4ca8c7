"""MI355X (gfx950) CSR sparse matrix-vector product: y <- alpha*A*x + beta*y.

The package is a C-ABI shared library (csrc/, include/spmv_mi355.h) and this thin ctypes
binding.  PyTorch is only used by callers for device memory and streams.
"""
from .spmv import *  # noqa: F401,F403
from .spmv import (CsrMatrix, SpmvError, check, library_path, spmv_analysis_host_t, spmv_analysis_info_t,
                   spmv_analyze_params_t)
