"""libgsa: Gated Slot Attention (arXiv 2409.07146) as hand-written HIP kernels for MI355X.

The package is a thin binding over the C-ABI library `libgsa.so` built from `csrc/`.
"""
from .api import (GsaError, alloc_decode_workspace, alloc_workspace, gsa_bwd, gsa_decode_step,  # noqa: F401
                  gsa_decode_step_static, gsa_decode_workspace_bytes, gsa_fwd, gsa_fwd_act,
                  gsa_profile_copy, gsa_profile_enable, gsa_profile_read, gsa_profile_reset, gsa_workspace_bytes,
                  make_problem)
from .autograd import gsa_attention  # noqa: F401,E402
