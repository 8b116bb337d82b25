"""MI355X-native batched top-k maximum-inner-product retrieval (the retrieval step of
an LLM search agent): exact flat scan and approximate graph beam search, as
hand-written HIP kernels behind the C ABI of include/ann.h."""
from .binding import (AnnError, ann_flat_search, ann_flat_search_typed, ann_flat_workspace_bytes,  # noqa: F401
                      ann_gather_ids, ann_graph_nonstall_workspace_bytes, ann_graph_search,
                      ann_graph_search_entries_typed, ann_graph_search_multi_typed, ann_graph_search_nonstall_typed,
                      ann_flat_search_static,
                      ann_graph_search_typed, ann_last_error, ann_measure_mfma_rate, ann_priority_order, ann_register_corpus,
                      ann_release_workspace, ann_set_workspace, ann_timing_enable, ann_timing_read, ann_timing_read_each, ann_set_default_dtype, ann_unregister_corpus, ann_version)
