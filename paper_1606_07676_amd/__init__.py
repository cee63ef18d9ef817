"""MI355X-native isomorphic sparse all-to-all / allgather on a virtual torus.

Thin Python binding over the C ABI of libiso.so (include/iso.h).  Every step of
the collectives runs in the library's HIP kernels; this package only marshals
arguments.  PyTorch is used by callers for device memory and streams.
"""
from .binding import (  # noqa: F401
    IsoError, load_library, library_path,
    ISO_OP_ALLTOALL, ISO_OP_ALLGATHER,
    ISO_ALG_COMBINED, ISO_ALG_COMBINED_BYDIM, ISO_ALG_SX_ROUNDS, ISO_ALG_SX_FUSED, ISO_ALG_ONEHOP,
    ISO_ALG_COMBINED_STAGED,
    ISO_BUF_SEND, ISO_BUF_RECV, ISO_BUF_WORK,
    ISO_LAYOUT_RANK_MAJOR, ISO_LAYOUT_SLOT_MAJOR, ISO_SX_LAUNCHES, ISO_SX_FUSED, ISO_GRAPH_OFF, ISO_GRAPH_CHAIN, ISO_GRAPH_BRANCHES,
    iso_alltoall_workspace_bytes, iso_allgather_workspace_bytes,
    iso_neighbor_alltoall_sx_init, iso_neighbor_allgather_sx_init,
    ISO_ROUND_SHIFT, ISO_ROUND_SELF, ISO_ROUND_VECTOR, ISO_ROUND_DELIVER,
    ISO_SUCCESS, ISO_ERR_ARG, ISO_ERR_OVERLAP, ISO_ERR_WORKSPACE, ISO_ERR_HIP,
    ISO_ERR_NOMEM, ISO_ERR_TOO_LARGE, ISO_ERR_POINTER, ISO_ERR_SCRATCH, ISO_MAX_DIMS,
    ISO_NOALLOC_SCRATCH_BYTES, ISO_NOALLOC_TABLE_BYTES, iso_neighbor_alltoall_noalloc,
    Comm, Plan, Request,
    iso_neighborhood_create, iso_neighborhood_create_mesh, iso_neighborhood_info, iso_neighborhood_free,
    iso_plan_create, iso_plan_info, iso_plan_round, iso_plan_entries, iso_plan_free,
    iso_workspace_bytes, iso_neighbor_alltoall_init, iso_neighbor_allgather_init,
    iso_neighbor_alltoall_init_layout, iso_neighbor_allgather_init_layout,
    iso_workspace_bytes_v, iso_neighbor_alltoallv_init, iso_neighbor_allgatherv_init,
    iso_neighbor_alltoallw_init, iso_neighbor_allgatherw_init,
    iso_neighbor_alltoallv_init_layout, iso_neighbor_allgatherv_init_layout,
    iso_start, iso_start_range, iso_request_set_graph, iso_wait, iso_request_info, iso_request_plan, iso_request_free,
    iso_error_string, iso_last_hip_error, iso_copy_reference,
)
