"""Seeded synthetic inputs for the sparse-convolution layer.

This module only *draws* data: occupancy patterns, feature values and filter
weights.  It contains none of the layer's arithmetic (no convolution, no
selection, no pooling) so that both the CPU oracle's tests and the HIP path's
tests can import it without sharing any method code.

The inputs stand in for the workloads the paper measures on (thresholded
hand-written digits in 2-D; voxelised CAD models / indoor scans in 3-D, whose
occupied voxels form thin surfaces with density about 1/r .. 3/r, Fig. 1 and
Sec. 4.1).  No item of any dataset is reproduced: strokes and shells are drawn
from a seeded generator.
"""
from .generators import (  # noqa: F401
    CONFIGS,
    LayerSpec,
    Workload,
    make_config,
    make_filter,
    make_octnet3_stack,
    make_paper_runtime,
    random_sparse_sites,
    shell_volume,
    stroke_image,
    sort_rows,
)
