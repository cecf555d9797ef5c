"""MI355X-native AdaScale SGD step: thin Python binding over the C-ABI library
`libadascale.so` (hand-written HIP for gfx950).  All arithmetic runs in the library's
kernels; this package only marshals arguments."""
from .binding import (AdaScale, AdaScaleError, State, Tuning, BF16, COOPERATIVE_LAUNCH, EST_NORM_RATIO, F32, LAGGED_R,
                      NO_POINTER_CHECK, FORCE_NONE, FORCE_GENERAL, FORCE_FUSED, FORCE_STREAMING, library_path,
                      load_library, step_flat)

from .driver import run_until_done

__all__ = ["run_until_done", "AdaScale", "AdaScaleError", "State", "Tuning", "F32", "BF16", "LAGGED_R", "EST_NORM_RATIO",
           "NO_POINTER_CHECK", "COOPERATIVE_LAUNCH", "FORCE_NONE", "FORCE_GENERAL", "FORCE_FUSED", "FORCE_STREAMING",
           "library_path", "load_library", "step_flat"]
