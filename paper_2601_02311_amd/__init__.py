"""Placement-sharded optimizer step for MI355X: Python binding of the C ABI.

The work is done by ``libps_step.so`` (hand-written HIP for gfx950, built from
``csrc/``); this package only marshals arguments.  Device buffers are passed
as integer addresses (``tensor.data_ptr()``) and streams as integer handles
(``torch.cuda.current_stream().cuda_stream``).
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
