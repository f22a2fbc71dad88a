"""MI355X-native batched integer max-flow feasibility checks (the data-parallel hot path of
ForestColl's schedule generator, arXiv 2402.06787).

The product is the C-ABI library `libfcmaxflow.so` (HIP kernels for gfx950 + host driver);
this package is its thin Python binding.  Build it with `python -m paper_2402_06787_amd.build`.
"""
from .binding import (FcError, Graph, GraphInfo, fc_options, fc_stats, fc_rational, load_library, strerror,
                      fc_graph_build, fc_graph_upload, fc_graph_upload_with_spares, fc_graph_update_arcs, fc_graph_sink_table, fc_graph_info, fc_graph_csr, fc_graph_set_source_weights,
                      fc_maxflow_batch_workspace_bytes, fc_maxflow_batch, fc_maxflow_batch_static,
                      FC_MAXFLOW_BATCH_STATIC_MAX_PROBLEMS,
                      fc_feasible_workspace_bytes, fc_feasible, fc_opt_throughput_search,
                      fc_search_with_verdicts, fc_maxflow_batch_floor, fc_feasible_floor, fc_fixed_k_search,
                      fc_fixed_k_search_with_verdicts, fc_split_gamma_workspace_bytes, fc_split_gamma_batch, fc_remove_switches,
                      fc_tree_mu_batch, fc_construct_trees, LIB_PATH, EXPORTED)
from .binding import (FC_OK, FC_EINVAL, FC_EOVERFLOW, FC_EDISCONNECTED, FC_ENOMEM, FC_EWORKSPACE, FC_EDEVICE,
                      FC_ENOCONVERGE, FC_EUNSUPPORTED, FC_FLOW_INVALID, FC_FLOW_NOCONVERGE, FC_FLOW_UNSUPPORTED,
                      FC_GAMMA_INVALID, FC_MU_INVALID)
