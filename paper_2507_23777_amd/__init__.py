"""MI355X-native multi-head speculative decoding step (XSpecMesh, arXiv 2507.23777).

The product is ``libxsm.so`` (hand-written gfx950 HIP kernels behind the C ABI of
``include/xsm.h``); this package is its thin ctypes binding.  PyTorch is used
for device memory and streams only.  There is no CPU fallback: every call
raises if the library has not been built (``python -m paper_2507_23777_amd.build``).
"""
from .xsm import (XSM_BF16, XSM_F32, Engine, StepBuffers, XsmError, lib, xsm_batch, xsm_config,
                  xsm_verify_params)
from .metrics import step_compression_ratio, speedup
from .batcher import Batcher, Request

__all__ = ["Engine", "StepBuffers", "XsmError", "lib", "xsm_batch", "xsm_config",
           "xsm_verify_params", "XSM_F32", "XSM_BF16", "step_compression_ratio", "speedup",
           "Batcher", "Request"]
