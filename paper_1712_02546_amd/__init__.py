"""MI355X-native convolution over a kernel slice (arXiv 1712.02546, Section 4.1.2).

Thin Python front end of libconvslice.so; see include/convslice.h for the ABI.
"""
from .binding import (CONV_BF16, CONV_F32, PASS_BWD_DATA, PASS_BWD_WEIGHT, PASS_FWD, ConvDesc,
                      ConvError, conv_bwd_data, conv_bwd_weight, conv_fwd, conv_output_dims, conv_probe_next_call,
                      conv_workspace_bytes, load, status_string)

__all__ = ["CONV_BF16", "CONV_F32", "PASS_BWD_DATA", "PASS_BWD_WEIGHT", "PASS_FWD", "ConvDesc",
           "ConvError", "conv_bwd_data", "conv_bwd_weight", "conv_fwd", "conv_output_dims", "conv_probe_next_call",
           "conv_workspace_bytes", "load", "status_string"]
