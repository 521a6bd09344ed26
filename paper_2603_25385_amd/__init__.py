"""GlowQ group forward for AMD MI355X: thin Python access to the C-ABI library.

    R = X B^T once per input-sharing group, Y_i = X dequant(W_q,i)^T + R A_i^T
    for every module of the group, with the GlowQ-S restore mask (paper Sec. 3.3).

The work is done by hand-written HIP kernels behind `include/glowq.h`; this
package only marshals arguments.  Importing it without a built library raises.
"""
from .binding import *  # noqa: F401,F403
from .binding import EXPORTED, GlowqError, glowq_module, glowq_unit, make_module, make_unit, pack_mask, pack_units  # noqa: F401
