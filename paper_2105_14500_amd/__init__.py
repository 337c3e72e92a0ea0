"""MI355X-native per-processor compute of a Tesseract [q,q,d]-partitioned linear layer.

`binding` is a thin ctypes layer over the C ABI in include/tesseract.h (argument
marshalling only); `partition` holds the host-side block views of Alg. 3 used to
emulate a whole processor grid on one GPU.
"""
from . import binding, partition  # noqa: F401
from .binding import (TessDesc, TessError, linear_fwd, linear_bwd_dx, linear_bwd_dw,  # noqa: F401
                      linear_bwd_dx_act, linear_bwd_dw_bias, linear_bwd_dx_step, linear_bwd_dw_step,
                      workspace_bytes, plan, desc_check, block_shape, status_string, version)
