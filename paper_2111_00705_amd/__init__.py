"""MI355X (gfx950) library for communication-compressed distributed AMSGrad (error feedback and CD-Adam).

The work is in csrc/ (hand-written HIP kernels behind the C ABI of
include/comp_ams.h); this package only builds and binds it.
"""
from .binding import (BLOCKSIGN, EDEVICE, EINVAL, ENOMEM, ESTATE, EXPORTS, METHOD_CD, METHOD_EF, METHOD_NAIVE, METHOD_NONE, OK, RANDK, TOPK, CompAms,
                      CompAmsError, lib, probe_copy, probe_update)

__all__ = ["CompAms", "CompAmsError", "lib", "probe_copy", "probe_update", "TOPK", "BLOCKSIGN", "RANDK", "METHOD_EF", "METHOD_CD", "METHOD_NAIVE", "METHOD_NONE", "EXPORTS",
           "OK", "EINVAL", "ENOMEM", "EDEVICE", "ESTATE"]
