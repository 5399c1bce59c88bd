"""MI355X-native GCN layer path (aggregation SpMM + update GEMMs, forward and backward).

Thin Python binding over the C ABI of ``libmixgcn.so`` (see ``include/mixgcn.h``).  Nothing
is computed in Python: the wrappers only marshal pointers, sizes and streams.  torch is used
for device memory and streams.  There is no CPU fallback: a missing library is an error.
"""
from .binding import (  # noqa: F401
    AGG_FIRST, UPDATE_FIRST, BF16, F32, NORM_SYM, NORM_MEAN, NORM_SUM, EPI_RELU, EPI_ACCUMULATE, ARITH_FP32, ARITH_BF16X3, OP_DGRAD, OP_FWD, OP_FWD_RELU, OP_WGRAD, SYMMETRIZE, ADD_SELF_LOOPS,
    BUILD_TRANSPOSE, INPUT_ON_HOST, Graph, LayerDesc, MixGCNError, Pipeline, aggregate, aggregate_masked,
    aggregate_scratch_bytes, aggregate_static, graph_reserve_streams,
    apply_bitmap,
    backward_pipelined, bandwidth, build_csr, dropout_bitmap, forward_pipelined, pipeline_window,
    cu_subset_stream,
    layer_bwd, layer_fwd, lib_path, load_library, measure_peaks, normalize, permute_rows, pipeline_stages, relabel_edges,
    relu_bitmap, reorder_rcm, set_aggregate_whole_rows, set_update_arith, softmax_xent, update, version,
)
from .model import GCNDropoutStep, GCNStep, GINStep, SAGEStep  # noqa: F401
