"""MaxK-GNN aggregation hot path on AMD MI355X: thin Python binding of libmaxk.

Argument marshalling only -- every step (top-k/CBSR, forward SpGEMM, backward
SSpMM, dense SpMM baseline, graph preprocessing) runs in the HIP kernels behind
the C ABI declared in ``include/maxk.h``.  PyTorch supplies device memory and
the stream, nothing else.  There is no CPU or eager fallback: if ``libmaxk.so``
is missing or a call fails, an exception is raised.
"""
from .binding import (  # noqa: F401
    BWD_AUTO,
    BWD_EXPAND_REDUCE,
    BWD_PULL_CSC,
    BWD_PUSH_CSR,
    BWD_SLAB_PULL,
    BWD_TILED,
    VALUE_BF16,
    VALUE_F16,
    VALUE_F32,
    MaxKError,
    MaxKGraph,
    index_dtype,
    lib_path,
    load_library,
    maxk_cbsr_scatter,
    maxk_graph_create,
    maxk_graph_destroy,
    maxk_spgemm_fwd,
    maxk_spgemm_fwd_narrow,
    maxk_spgemm_fwd_noalloc,
    maxk_sspmm_bwd,
    maxk_sspmm_bwd_narrow,
    maxk_topk_cbsr,
    maxk_topk_cbsr_narrow,
    spmm_baseline,
)
from .autograd import MaxKAggregate, maxk_aggregate  # noqa: E402,F401
