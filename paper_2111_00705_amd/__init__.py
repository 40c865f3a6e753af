"""MI355X (gfx950) library for error-feedback-compressed distributed AMSGrad.

The work is in csrc/ (hand-written HIP kernels behind the C ABI of
include/comp_ams.h); this package only builds and binds it.
"""
from .binding import (BLOCKSIGN, EDEVICE, EINVAL, ENOMEM, ESTATE, EXPORTS, OK, TOPK, CompAms, CompAmsError,
                      lib, probe_copy)

__all__ = ["CompAms", "CompAmsError", "lib", "probe_copy", "TOPK", "BLOCKSIGN", "EXPORTS", "OK", "EINVAL", "ENOMEM",
           "EDEVICE", "ESTATE"]
