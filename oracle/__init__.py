"""CPU oracle of the partition-n-reduce shard path (arXiv 1807.08887).

TEST INFRASTRUCTURE.  Only tests, the smoke check and the bench's cpu_baseline leg may
import this package; the product path (paper_1807_08887_amd) never does, and this package
never imports the product.  `regions` holds the integer range/region definitions and the
fetch; `ops` wraps the fp64 loop nests of tofu_oracle.c.
"""
from . import regions  # noqa: F401
from .ops import (build, conv1d_box, conv2d_box, conv2d_pts, dgrad_box, dgrad_pts, lstm_cell, matmul_box, matmul_pts, reduce, reduce_op, threads,  # noqa: F401
                  wgrad_box, wgrad_pts)
