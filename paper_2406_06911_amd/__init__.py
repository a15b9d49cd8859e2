"""MI355X-native asynchronous denoising (AsyncDiff, arXiv 2406.06911): thin Python binding over the
C ABI in include/asyncdiff.h.  All arithmetic runs in the HIP library; this package only marshals
arguments and uses PyTorch for device memory and streams."""
from .binding import (AD_BF16, AD_DDIM, AD_EULER, AD_F32, AD_BETA_LINEAR, AD_BETA_SCALED_LINEAR, AsyncDiff, AsyncDiffError,
                      UNetCfg, balance_cuts, lib, lib_path)

__all__ = ["balance_cuts", "AsyncDiff", "AsyncDiffError", "UNetCfg", "lib", "lib_path", "AD_F32", "AD_BF16", "AD_DDIM", "AD_EULER",
           "AD_BETA_LINEAR", "AD_BETA_SCALED_LINEAR"]
