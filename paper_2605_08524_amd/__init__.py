"""MI355X-native block-level attention for one FCP worker: a C-ABI library of HIP
kernels (csrc/, include/fcp.h, include/fcp_sched.h) and a thin ctypes binding with the same names."""
from .binding import (  # noqa: F401
    FCP_FLAG_DIRECT_SINGLE, FCP_FLAG_O_F32, FCP_FLAG_GRAD_BF16, FCP_FLAG_PART_BF16, FCP_KIND_DIAG, FCP_KIND_FULL, FcpError, Problem, fcp_block_attn_bwd, fcp_block_attn_bwd_dkdv, fcp_block_attn_bwd_dq, fcp_block_attn_bwd_dq_d, fcp_bwd_preprocess,
    fcp_block_attn_fwd, fcp_block_attn_fwd_out, fcp_device_info, fcp_last_error, fcp_mfma_probe, fcp_merge_partials, fcp_plan_blocks,
    fcp_queue_build, fcp_workspace_bytes,
    FCP_ERR_INFEASIBLE, fcp_assign_blocks, fcp_block_costs, fcp_coalesce_stages, fcp_comm_edges, fcp_pack_units, fcp_solve_matchings,
    fcp_worker_blocks,
)
