"""MI355X-native convolution over a kernel slice (arXiv 1712.02546, Section 4.1.2), the Eq. (1)
workload partition and the partitioned-layer driver (Section 3.1.1, Algorithm 1).

Thin Python front end of libconvslice.so; see include/convslice.h and include/convlayer.h for the ABI.
"""
from .binding import (CONV_BF16, CONV_F32, MAX_DEVICES, NOALLOC_MAX_WORKSPACE, PASS_BWD_DATA, PASS_BWD_WEIGHT, PASS_FWD, ConvDesc,
                      ConvError, conv_bwd_data, conv_bwd_weight, conv_calibrate, conv_calibrate_workspace_bytes,
                      conv_comm_elements, conv_comm_elements_partition, conv_scaling_estimate,
                      conv_fwd, conv_fwd_noalloc, conv_layer_bwd_data, conv_layer_bwd_weight, conv_layer_fwd,
                      conv_layer_workspace_bytes, conv_output_dims, conv_pass_path, conv_partition, conv_partition_estimate,
                      conv_probe_next_call, conv_workspace_bytes, load, net_fc_bwd, net_fc_fwd, net_norm_bwd,
                      net_norm_fwd, net_pool_bwd, net_pool_fwd, net_sgd_update, net_softmax_loss_bwd,
                      net_softmax_loss_fwd, pass_mask, status_string)

__all__ = ["CONV_BF16", "CONV_F32", "MAX_DEVICES", "NOALLOC_MAX_WORKSPACE", "PASS_BWD_DATA", "PASS_BWD_WEIGHT", "PASS_FWD", "ConvDesc",
           "ConvError", "conv_bwd_data", "conv_bwd_weight", "conv_calibrate", "conv_calibrate_workspace_bytes",
           "conv_comm_elements", "conv_comm_elements_partition", "conv_scaling_estimate",
           "conv_fwd", "conv_fwd_noalloc", "conv_layer_bwd_data", "conv_layer_bwd_weight", "conv_layer_fwd",
           "conv_layer_workspace_bytes", "conv_output_dims", "conv_pass_path", "conv_partition", "conv_partition_estimate",
           "conv_probe_next_call", "conv_workspace_bytes", "load", "net_fc_bwd", "net_fc_fwd", "net_norm_bwd",
           "net_norm_fwd", "net_pool_bwd", "net_pool_fwd", "net_sgd_update", "net_softmax_loss_bwd",
           "net_softmax_loss_fwd", "pass_mask", "status_string"]
