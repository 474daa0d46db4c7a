"""tjnvfp4: NVFP4 fully-quantized linear layer (TetraJet-v2, arXiv 2510.27527) for MI355X.

The product is the C-ABI library ``libtjnvfp4.so`` (``include/tjnvfp4.h``); this package holds
its HIP sources (``csrc/``), the build step (``build.py``) and a thin ctypes binding
(``binding.py``) with the same call names.
"""
from . import binding  # noqa: F401
from .binding import (NVFP4Error, NVFP4Tensor, alloc_nvfp4, alloc_workspace, amax_bf16, gemm_nt, gemm_nt_static,  # noqa: F401
                      linear_bwd_dw,
                      linear_bwd, linear_bwd_dx, linear_fwd, osci_select, osci_suppress, osci_suppress_sparse, osci_update, osci_update_sparse, outctl_bwd, outctl_fwd, quantize, quantize_dual, stream_key, workspace_bytes)
