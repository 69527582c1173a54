"""MI355X-native classifier-layer hot path of ASTRA (arXiv 2409.20156).

The compute lives in libastra_xc.so (hand-written HIP for gfx950, C ABI in
include/astra_xc.h).  `binding` marshals torch device tensors into that ABI;
`synth` makes the seeded synthetic inputs.  Nothing here falls back to another
implementation: calls raise if the library is not built or no GPU is present.
"""
from .binding import (XC_BF16, XC_F32, XC_LOSS_BCE, XC_LOSS_SOFTMAX, XcError, load_library,
                      mine_negatives, mine_workspace, sample_negatives, sample_negatives_mixture, sample_negatives_pps,
                      step_workspace, xc_step, xc_step_static)

__all__ = ["XC_BF16", "XC_F32", "XC_LOSS_BCE", "XC_LOSS_SOFTMAX", "XcError", "load_library",
           "mine_negatives", "mine_workspace", "sample_negatives", "sample_negatives_mixture", "sample_negatives_pps", "step_workspace",
           "xc_step", "xc_step_static"]
