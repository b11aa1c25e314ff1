"""SDGP backward-data path for AMD MI355X (gfx950).

Structured Data Gradient Pruning (arXiv 2202.00774) keeps n of every m channels
of the output data gradient (Alg. 1, Sec. III-B) and computes the input data
gradient from the pruned tensor (Fig. 1-3).  The work is done by hand-written
HIP kernels behind a C ABI (``include/sdgp.h``); this package is the thin Python
binding over it.  There is no CPU fallback: without the built library every
call raises.
"""
from .binding import (BF16, F32, GREEDY, GREEDY_ADJUSTED, RANDOM, SdgpError, conv_bwd_data_workspace,
                      library_path, sdgp_channel_scales, sdgp_conv_bwd_data, sdgp_conv_bwd_data_channel_rescaled,
                      sdgp_conv_bwd_data_compact, sdgp_conv_bwd_data_grouped, sdgp_conv_bwd_data_noalloc, sdgp_conv_bwd_weight, sdgp_conv_fwd, sdgp_linear_bwd_data, sdgp_linear_bwd_data_channel_rescaled, sdgp_peak_probe, sdgp_prune,
                      sdgp_prune_channel_rescaled, sdgp_scale_filter, status_string, version)

__all__ = ["BF16", "F32", "GREEDY", "GREEDY_ADJUSTED", "RANDOM", "SdgpError", "conv_bwd_data_workspace",
           "library_path", "sdgp_channel_scales", "sdgp_conv_bwd_data", "sdgp_conv_bwd_data_channel_rescaled",
           "sdgp_conv_bwd_data_compact", "sdgp_conv_bwd_data_grouped", "sdgp_conv_bwd_data_noalloc", "sdgp_conv_bwd_weight", "sdgp_conv_fwd", "sdgp_linear_bwd_data", "sdgp_linear_bwd_data_channel_rescaled", "sdgp_peak_probe", "sdgp_prune",
           "sdgp_prune_channel_rescaled", "sdgp_scale_filter", "status_string", "version"]
