"""MI355X-native block-level attention for one FCP worker: a C-ABI library of HIP
kernels (csrc/, include/fcp.h, include/fcp_sched.h) and a thin ctypes binding with the same names.

The binding (and with it libfcp.so) is loaded on the first use of one of its names, not when the
package is imported: `paper_2605_08524_amd.workloads`, the seeded input generators that feed both
this library and the CPU oracle, must be importable where the library has not been built.  There is
no fallback: touching any binding name without a built libfcp.so raises ImportError."""
import importlib

_BINDING_NAMES = (
    "FCP_FLAG_DIRECT_SINGLE", "FCP_FLAG_O_F32", "FCP_FLAG_GRAD_BF16", "FCP_FLAG_PART_BF16", "FCP_FLAG_BWD_SPILL_DS", "FCP_FLAG_RUNNING_MERGE",
    "FCP_KIND_DIAG", "FCP_KIND_FULL", "FCP_KIND_PACKED_FULL", "FCP_KIND_PACKED_DIAG", "FCP_ERR_INFEASIBLE", "FcpError", "Problem",
    "fcp_plan_blocks", "fcp_plan_blocks_packed", "fcp_stage_tables", "fcp_workspace_bytes", "fcp_queue_build", "fcp_block_attn_fwd", "fcp_block_attn_fwd_out",
    "fcp_block_attn_fwd_static",
    "fcp_merge_partials", "fcp_block_attn_bwd", "fcp_bwd_preprocess", "fcp_block_attn_bwd_dkdv",
    "fcp_block_attn_bwd_dq", "fcp_block_attn_bwd_dq_d", "fcp_block_attn_bwd_dq_ds", "fcp_device_info", "fcp_last_error", "fcp_mfma_probe", "fcp_mfma_valu_probe", "fcp_lds_probe", "fcp_atomic_probe",
    "fcp_assign_blocks", "fcp_block_costs", "fcp_coalesce_stages", "fcp_comm_edges", "fcp_pack_units",
    "fcp_solve_matchings", "fcp_worker_blocks",
)


def __getattr__(name):
    if name in _BINDING_NAMES or name == "binding":
        binding = importlib.import_module(".binding", __name__)
        if name == "binding":
            return binding
        return getattr(binding, name)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")


def __dir__():
    return sorted(list(globals()) + list(_BINDING_NAMES))
