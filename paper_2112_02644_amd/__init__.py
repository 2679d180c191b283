"""MI355X (gfx950) library for the batched hot path of semantic-memory CNN inference
(arXiv 2112.02644): encode -> lookup -> exit/compact per exit point, memory update between
batches.  The arithmetic lives in the HIP library libsmtm.so; this package only marshals
arguments to its C ABI (include/smtm.h)."""
from .smtm import (Smtm, SmtmConfig, SmtmError, load_library, F16, F32,
                   SCORE_AUTO, SCORE_FP32, SCORE_MFMA)

__all__ = ["Smtm", "SmtmConfig", "SmtmError", "load_library", "F16", "F32",
           "SCORE_AUTO", "SCORE_FP32", "SCORE_MFMA"]
