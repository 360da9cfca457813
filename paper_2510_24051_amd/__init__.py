"""MI355X-native hot path of a programmable LLM serving system's inference layer: the batched
`forward` handler and the `get_next_dist` handler, as hand-written HIP kernels behind a C ABI
(include/pie_mi355.h).  This package is the thin Python binding: argument marshalling only."""
from .binding import (PIE_N_STAGES, STAGE_NAMES, TAP_ACT, TAP_ATTN, TAP_LOGITS, TAP_Q, TAP_RESID, Pie, PieBatch,
                      PieError, lib_path, load_library)

__all__ = ["Pie", "PieBatch", "PieError", "load_library", "lib_path", "STAGE_NAMES", "PIE_N_STAGES",
           "TAP_Q", "TAP_ATTN", "TAP_RESID", "TAP_ACT", "TAP_LOGITS"]
