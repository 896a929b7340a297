"""MI355X-native shard hot path of Tofu's partition-n-reduce method (arXiv 1807.08887).

A thin Python binding over the C ABI declared in include/tofu.h.  Every step of the path runs
in the HIP kernels of libtofu.so; Python only marshals arguments.  PyTorch is used for device
memory and streams.
"""
from .binding import (TOFU_MAX_DIMS, OpDesc, Region, Split, Tensor, TofuError, conv2d_desc, dgrad_desc, last_error, lstm_cell_desc, shard_lstm_cell, lib_path,  # noqa: F401
                      load, matmul_desc, op_regions, partition_reduce, probe_copy, probe_mfma, probe_read, probe_stream, region_fetch, shard_conv2d, shard_conv2d_dgrad, shard_conv2d_fused, shard_conv2d_wgrad,
                      shard_matmul, shard_range, tensor, wgrad_desc, workspace_bytes, partition_reduce_scatter, shard_matmul_accumulate,
                      shard_conv2d_accumulate, shard_conv2d_wgrad_accumulate, shard_conv2d_dgrad_accumulate, conv1d_desc, shard_conv1d,
                      shard_conv1d_accumulate, shard_matmul_noalloc, OP_CONV1D, CONV1D_DIM_B, CONV1D_DIM_CO, CONV1D_DIM_X, CONV1D_DIM_CI)
from .binding import (LSTM_DIM_B, LSTM_DIM_H, OP_LSTM_CELL, ORDER_LINEAR, ORDER_TREE, REDUCE_MAX, REDUCE_MIN, REDUCE_PROD, REDUCE_SUM,  # noqa: F401
                      DGRAD_DIM_CI, DGRAD_DIM_CO, DGRAD_DIM_H, DGRAD_DIM_N, DGRAD_DIM_W, OP_CONV2D_DGRAD,  # noqa: F401
                      CONV_DIM_CI, CONV_DIM_CO, CONV_DIM_H, CONV_DIM_N, CONV_DIM_W, MM_DIM_K, MM_DIM_M, MM_DIM_N,  # noqa: F401
                      OP_CONV2D, OP_CONV2D_WGRAD, OP_MATMUL, WGRAD_DIM_CI, WGRAD_DIM_CO, WGRAD_DIM_N)
