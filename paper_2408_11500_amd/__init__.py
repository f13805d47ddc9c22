"""MI355X-native hot path of SliceGCN (arXiv 2408.11500): HIP kernels behind a C ABI.

``binding`` mirrors the C entry points of ``include/slicegcn.h`` one to one; ``build`` compiles
the library.  Importing the package does not load the library; the first call does, and it
raises if the library is missing (there is no CPU path).
"""
from . import binding  # noqa: F401
from .binding import (ACT_NONE, ACT_RELU, ADD_SELF_LOOPS, SYMMETRIZE, Graph, SliceGCNError,  # noqa: F401
                      slicegcn_build_norm_csr, slicegcn_concat, slicegcn_concat_bwd,
                      slicegcn_concat_bwd_workspace_bytes, slicegcn_layer_bwd,
                      slicegcn_layer_bwd_workspace_bytes, slicegcn_layer_fwd,
                      slicegcn_layer_fwd_workspace_bytes, slicegcn_profile_begin, slicegcn_profile_reserve,
                      slicegcn_profile_end, slicegcn_scale_rows, slicegcn_slice_feature,
                      slicegcn_slice_strategy, slicegcn_spmm_slice, slicegcn_spmm_workspace_bytes)
