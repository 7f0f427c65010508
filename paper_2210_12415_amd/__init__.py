"""MI355X-native tensor operators under explicit data layouts (conv2d, gemm,
layout_transform, joint layout/tile tuning) — thin ctypes binding over the
C ABI in include/alt.h.  All computation happens in libalt.so's HIP kernels;
this package only marshals arguments.  There is no CPU fallback: importing
works without a GPU (layout index math is host code), but every call that
needs a kernel raises AltError when the library or the device is missing."""
from .binding import (AltError, Handle, Layout, ConvDesc, GemmDesc, TuneOpts, TuneReport,
                      ChainPlan, Prim, Peaks, F32, BF16, EPI_BIAS, EPI_RELU,
                      layout_parse, layout_from_prims, layout_physical_shape, layout_offset,
                      layout_index_of, plan_chain, split, reorder, fuse, version, lib,
                      conv_desc, gemm_desc, exported_symbols, library_path)
