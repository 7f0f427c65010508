"""MI355X-native tensor operators under explicit data layouts (conv2d, gemm,
layout_transform, joint layout/tile tuning) — thin ctypes binding over the
C ABI in include/alt.h.  All computation happens in libalt.so's HIP kernels;
this package only marshals arguments.  There is no CPU fallback: importing
works without a GPU (layout index math is host code), but every call that
needs a kernel raises AltError when the library or the device is missing."""
import os as _os

# Kernel arguments in device memory (HIP's default is host memory, which costs
# every launch of these short kernels microseconds of host-link latency).
# Only effective if set before the HIP runtime starts in this process.
_os.environ.setdefault("HIP_FORCE_DEV_KERNARG", "1")

from .binding import (AltError, Handle, Layout, ConvDesc, Conv3dDesc, ConvCall, GemmDesc, TuneOpts, TuneReport,
                      ChainPlan, GraphNode, GraphPlan, NODE_CONV, NODE_ADD, Prim, Peaks, F32, BF16, EPI_BIAS, EPI_RELU,
                      SplitkStatus, TransformPlan, layout_parse, layout_from_prims, layout_physical_shape, layout_offset,
                      layout_index_of, plan_chain, plan_graph, graph_node, unfold_shape, split, reorder, fuse, version, lib,
                      conv_desc, conv3d_desc, gemm_desc, exported_symbols, library_path)
