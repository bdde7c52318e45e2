"""ctypes binding of libfcp.so: same names as the C ABI, argument marshalling only.

Every step of the path runs inside the library's kernels.  Tensors may be
anything exposing ``data_ptr()`` (PyTorch device tensors: PyTorch is used for
device memory and streams only) or plain integers holding device addresses.
There is no fallback: if the shared library is missing the import of this module
fails.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# FCP_LIB_PATH (debugging only): another build of the same library, e.g. the one with host-side sanitizers
LIB_PATH = os.environ.get("FCP_LIB_PATH") or os.path.join(_HERE, "libfcp.so")

FCP_OK = 0
FCP_ERR_INVALID_ARG = -1
FCP_ERR_BUFFER_TOO_SMALL = -2
FCP_ERR_UNSUPPORTED = -3
FCP_ERR_HIP = -4
FCP_ERR_INFEASIBLE = -5
FCP_KIND_FULL, FCP_KIND_DIAG, FCP_KIND_PACKED_FULL, FCP_KIND_PACKED_DIAG = 0, 1, 2, 3
FCP_FLAG_O_F32 = 1
FCP_FLAG_DIRECT_SINGLE = 2
FCP_FLAG_PART_BF16 = 4
FCP_FLAG_GRAD_BF16 = 8
FCP_FLAG_BWD_SPILL_DS = 16
FCP_FLAG_RUNNING_MERGE = 32

EXPORTS = (
    "fcp_plan_blocks", "fcp_plan_blocks_packed", "fcp_stage_tables", "fcp_workspace_bytes", "fcp_queue_build", "fcp_block_attn_fwd", "fcp_block_attn_fwd_out",
    "fcp_merge_partials", "fcp_block_attn_bwd", "fcp_bwd_preprocess", "fcp_block_attn_bwd_dkdv", "fcp_block_attn_bwd_dq",
    "fcp_block_attn_bwd_dq_d", "fcp_block_attn_bwd_dq_ds", "fcp_block_attn_fwd_static",
    "fcp_last_error", "fcp_device_info", "fcp_mfma_probe", "fcp_mfma_valu_probe", "fcp_lds_probe", "fcp_atomic_probe",
    "fcp_block_costs", "fcp_assign_blocks", "fcp_worker_blocks", "fcp_comm_edges", "fcp_solve_matchings",
    "fcp_coalesce_stages", "fcp_pack_units",
)


class FcpError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"fcp error {code}: {text}")
        self.code = code


class _Problem(C.Structure):
    _fields_ = [
        ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("block_size", C.c_int32),
        ("softmax_scale", C.c_float), ("flags", C.c_int32),
        ("n_kv_blocks", C.c_int32), ("n_q_blocks", C.c_int32), ("n_pairs", C.c_int32), ("n_slots", C.c_int32),
        ("n_slot_rows", C.c_int32),
        ("kv_blocks", C.c_void_p), ("q_blocks", C.c_void_p), ("pairs", C.c_void_p), ("slots", C.c_void_p),
        ("n_segments", C.c_int32), ("segments", C.c_void_p),
    ]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'). "
            "There is no CPU fallback.")
    # PyTorch ships a HIP runtime of its own.  Whichever copy is loaded first serves the whole process
    # (same SONAME), and tensors made by torch are only usable by this library if both talk to one
    # runtime: load torch's first when torch is installed.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(LIB_PATH)
    i32p = C.POINTER(C.c_int32)
    lib.fcp_plan_blocks.argtypes = [i32p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, i32p, C.c_int32,
                                    C.c_void_p, i32p, C.c_void_p, i32p, C.c_void_p, i32p, C.c_void_p, i32p, i32p]
    lib.fcp_plan_blocks_packed.argtypes = [i32p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, i32p, C.c_int32, i32p,
                                           C.c_void_p, i32p, C.c_void_p, i32p, C.c_void_p, i32p, C.c_void_p, i32p, i32p, C.c_void_p, i32p]
    lib.fcp_stage_tables.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int32,
                                     C.c_void_p, i32p, C.c_void_p, i32p, i32p]
    lib.fcp_workspace_bytes.argtypes = [C.POINTER(_Problem), C.POINTER(C.c_size_t)]
    lib.fcp_queue_build.argtypes = [C.POINTER(_Problem), C.c_void_p, C.c_size_t, C.c_void_p]
    lib.fcp_block_attn_fwd.argtypes = [C.POINTER(_Problem)] + [C.c_void_p] * 7
    lib.fcp_block_attn_fwd_out.argtypes = [C.POINTER(_Problem)] + [C.c_void_p] * 9
    lib.fcp_block_attn_fwd_static.argtypes = [C.POINTER(_Problem)] + [C.c_void_p] * 6
    lib.fcp_merge_partials.argtypes = [C.POINTER(_Problem)] + [C.c_void_p] * 6
    lib.fcp_block_attn_bwd.argtypes = [C.POINTER(_Problem)] + [C.c_void_p] * 11
    lib.fcp_bwd_preprocess.argtypes = [C.POINTER(_Problem)] + [C.c_void_p] * 5
    lib.fcp_block_attn_bwd_dkdv.argtypes = [C.POINTER(_Problem)] + [C.c_void_p] * 8
    lib.fcp_block_attn_bwd_dq.argtypes = [C.POINTER(_Problem)] + [C.c_void_p] * 7
    lib.fcp_block_attn_bwd_dq_d.argtypes = [C.POINTER(_Problem)] + [C.c_void_p] * 9
    lib.fcp_block_attn_bwd_dq_ds.argtypes = [C.POINTER(_Problem)] + [C.c_void_p] * 4
    i64p = C.POINTER(C.c_int64)
    lib.fcp_block_costs.argtypes = [i32p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, i32p]
    lib.fcp_pack_units.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, i32p]
    lib.fcp_assign_blocks.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_double, C.c_double, C.c_int64,
                                      C.c_double, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.fcp_worker_blocks.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, i32p]
    lib.fcp_comm_edges.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, i64p]
    lib.fcp_solve_matchings.argtypes = [C.c_void_p, C.c_int64, C.c_int32, i32p]
    lib.fcp_coalesce_stages.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, i32p]
    lib.fcp_last_error.restype = C.c_char_p
    lib.fcp_device_info.argtypes = [i32p, i32p, i32p]
    lib.fcp_mfma_probe.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    lib.fcp_mfma_valu_probe.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    lib.fcp_lds_probe.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.fcp_atomic_probe.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_void_p]
    for name in EXPORTS:
        if name != "fcp_last_error":
            getattr(lib, name).restype = C.c_int
    return lib


_lib = _load()


def _check(rc):
    if rc != FCP_OK:
        raise FcpError(rc, _lib.fcp_last_error().decode())


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(s):
    if s is None:
        return None
    if isinstance(s, int):
        return s
    return s.cuda_stream        # torch.cuda.Stream


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def fcp_last_error() -> str:
    return _lib.fcp_last_error().decode()


def fcp_plan_blocks(seq_lens, block_size, causal=1, coalesce=0, q_owned=None):
    """Returns dict(kv_blocks, q_blocks, pairs, slots: int32 [n,4]; n_slot_rows: int)."""
    sl = _i32(np.asarray(seq_lens).reshape(-1))
    qo = None if q_owned is None else _i32(np.asarray(q_owned).reshape(-1, 2))
    i32p = C.POINTER(C.c_int32)
    qo_p = None if qo is None else qo.ctypes.data_as(i32p)
    n_qo = 0 if qo is None else len(qo)
    counts = [C.c_int32(0) for _ in range(5)]
    args = [sl.ctypes.data_as(i32p), len(sl), int(block_size), int(causal), int(coalesce), qo_p, n_qo]
    _check(_lib.fcp_plan_blocks(*args, None, C.byref(counts[0]), None, C.byref(counts[1]), None,
                                C.byref(counts[2]), None, C.byref(counts[3]), C.byref(counts[4])))
    tabs = [np.zeros((max(1, c.value), 4), dtype=np.int32) for c in counts[:4]]
    _check(_lib.fcp_plan_blocks(*args, tabs[0].ctypes.data, C.byref(counts[0]), tabs[1].ctypes.data,
                                C.byref(counts[1]), tabs[2].ctypes.data, C.byref(counts[2]),
                                tabs[3].ctypes.data, C.byref(counts[3]), C.byref(counts[4])))
    tabs = [t[: c.value] for t, c in zip(tabs, counts[:4])]
    return dict(kv_blocks=tabs[0], q_blocks=tabs[1], pairs=tabs[2], slots=tabs[3], n_slot_rows=counts[4].value)


def fcp_plan_blocks_packed(seq_lens, block_size, causal=1, coalesce=0, q_owned=None, unit_of_block=None):
    """fcp_plan_blocks with every scheduling unit of two or more blocks (unit_of_block, from fcp_pack_units) as one
    packed block.  Returns the fcp_plan_blocks dict plus segments: int32 [n,4] = (kv_blk, seq, tok_off, tok_len)."""
    sl = _i32(np.asarray(seq_lens).reshape(-1))
    qo = None if q_owned is None else _i32(np.asarray(q_owned).reshape(-1, 2))
    ub = None if unit_of_block is None else _i32(np.asarray(unit_of_block).reshape(-1))
    i32p = C.POINTER(C.c_int32)
    args = [sl.ctypes.data_as(i32p), len(sl), int(block_size), int(causal), int(coalesce),
            None if qo is None else qo.ctypes.data_as(i32p), 0 if qo is None else len(qo),
            None if ub is None else ub.ctypes.data_as(i32p)]
    counts = [C.c_int32(0) for _ in range(6)]     # kv, q, pairs, slots, slot rows, segments

    def call(tabs):
        return _lib.fcp_plan_blocks_packed(*args, tabs[0], C.byref(counts[0]), tabs[1], C.byref(counts[1]), tabs[2], C.byref(counts[2]),
                                           tabs[3], C.byref(counts[3]), C.byref(counts[4]), tabs[4], C.byref(counts[5]))
    _check(call([None] * 5))
    sizes = [counts[i].value for i in (0, 1, 2, 3, 5)]
    tabs = [np.zeros((max(1, n), 4), dtype=np.int32) for n in sizes]
    _check(call([t.ctypes.data for t in tabs]))
    tabs = [t[:n] for t, n in zip(tabs, sizes)]
    return dict(kv_blocks=tabs[0], q_blocks=tabs[1], pairs=tabs[2], slots=tabs[3], n_slot_rows=counts[4].value, segments=tabs[4])


def fcp_stage_tables(plan, stage):
    """The plan restricted to one execution stage: returns (stage_plan, n_stages); stage_plan shares the block tables
    of `plan` and has n_slot_rows = all query tokens."""
    pairs, slots, qb = (_i32(plan[k]).reshape(-1, 4) for k in ("pairs", "slots", "q_blocks"))
    n_p, n_s, n_st = C.c_int32(0), C.c_int32(0), C.c_int32(0)
    args = [pairs.ctypes.data if len(pairs) else None, len(pairs), slots.ctypes.data if len(slots) else None, len(slots),
            qb.ctypes.data if len(qb) else None, len(qb), int(stage)]
    _check(_lib.fcp_stage_tables(*args, None, C.byref(n_p), None, C.byref(n_s), C.byref(n_st)))
    sp = np.zeros((max(1, n_p.value), 4), dtype=np.int32)
    ss = np.zeros((max(1, n_s.value), 4), dtype=np.int32)
    _check(_lib.fcp_stage_tables(*args, sp.ctypes.data, C.byref(n_p), ss.ctypes.data, C.byref(n_s), C.byref(n_st)))
    out = dict(plan)
    out.update(pairs=sp[: n_p.value], slots=ss[: n_s.value], n_slot_rows=int(qb[:, 3].sum()) if len(qb) else 0)
    return out, n_st.value


class Problem:
    """Owns the host tables of an fcp_problem and the ctypes struct pointing at them."""

    def __init__(self, plan, n_q_heads, n_kv_heads, head_dim, block_size, softmax_scale=0.0, flags=0):
        self.kv_blocks = _i32(plan["kv_blocks"]).reshape(-1, 4)
        self.q_blocks = _i32(plan["q_blocks"]).reshape(-1, 4)
        self.pairs = _i32(plan["pairs"]).reshape(-1, 4)
        self.slots = _i32(plan["slots"]).reshape(-1, 4)
        self.n_slot_rows = int(plan["n_slot_rows"])
        self.segments = _i32(plan["segments"]).reshape(-1, 4) if "segments" in plan else np.zeros((0, 4), dtype=np.int32)
        self.flags = int(flags)
        self.n_q_heads, self.n_kv_heads, self.head_dim = int(n_q_heads), int(n_kv_heads), int(head_dim)
        self.t_q = int(self.q_blocks[:, 3].sum()) if len(self.q_blocks) else 0
        self.t_kv = int(self.kv_blocks[:, 3].sum()) if len(self.kv_blocks) else 0
        self.c = _Problem(
            self.n_q_heads, self.n_kv_heads, self.head_dim, int(block_size), float(softmax_scale), int(flags),
            len(self.kv_blocks), len(self.q_blocks), len(self.pairs), len(self.slots), self.n_slot_rows,
            self.kv_blocks.ctypes.data if len(self.kv_blocks) else None,
            self.q_blocks.ctypes.data if len(self.q_blocks) else None,
            self.pairs.ctypes.data if len(self.pairs) else None,
            self.slots.ctypes.data if len(self.slots) else None,
            len(self.segments), self.segments.ctypes.data if len(self.segments) else None)

    @property
    def ref(self):
        return C.byref(self.c)


def fcp_workspace_bytes(problem: Problem) -> int:
    n = C.c_size_t(0)
    _check(_lib.fcp_workspace_bytes(problem.ref, C.byref(n)))
    return n.value


def fcp_queue_build(problem: Problem, workspace, workspace_bytes, stream=None):
    _check(_lib.fcp_queue_build(problem.ref, _ptr(workspace), int(workspace_bytes), _stream(stream)))


def fcp_block_attn_fwd(problem: Problem, q, k, v, o_part, lse_part, workspace, stream=None):
    _check(_lib.fcp_block_attn_fwd(problem.ref, _ptr(q), _ptr(k), _ptr(v), _ptr(o_part), _ptr(lse_part),
                                   _ptr(workspace), _stream(stream)))


def fcp_block_attn_fwd_out(problem: Problem, q, k, v, o_part, lse_part, o, lse, workspace, stream=None):
    _check(_lib.fcp_block_attn_fwd_out(problem.ref, _ptr(q), _ptr(k), _ptr(v), _ptr(o_part), _ptr(lse_part),
                                       _ptr(o), _ptr(lse), _ptr(workspace), _stream(stream)))


def fcp_block_attn_fwd_static(problem: Problem, q, k, v, o_part, lse_part, stream=None):
    _check(_lib.fcp_block_attn_fwd_static(problem.ref, _ptr(q), _ptr(k), _ptr(v), _ptr(o_part), _ptr(lse_part),
                                          _stream(stream)))


def fcp_merge_partials(problem: Problem, o_part, lse_part, o, lse, workspace, stream=None):
    _check(_lib.fcp_merge_partials(problem.ref, _ptr(o_part), _ptr(lse_part), _ptr(o), _ptr(lse),
                                   _ptr(workspace), _stream(stream)))


def fcp_block_attn_bwd(problem: Problem, q, k, v, o, lse, d_o, dq, dk, dv, workspace, stream=None):
    _check(_lib.fcp_block_attn_bwd(problem.ref, _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(d_o),
                                   _ptr(dq), _ptr(dk), _ptr(dv), _ptr(workspace), _stream(stream)))


def fcp_bwd_preprocess(problem: Problem, o, lse, d_o, workspace, stream=None):
    _check(_lib.fcp_bwd_preprocess(problem.ref, _ptr(o), _ptr(lse), _ptr(d_o), _ptr(workspace), _stream(stream)))


def fcp_block_attn_bwd_dkdv(problem: Problem, q, k, v, d_o, dk, dv, workspace, stream=None):
    _check(_lib.fcp_block_attn_bwd_dkdv(problem.ref, _ptr(q), _ptr(k), _ptr(v), _ptr(d_o),
                                        _ptr(dk), _ptr(dv), _ptr(workspace), _stream(stream)))


def fcp_block_attn_bwd_dq(problem: Problem, q, k, v, d_o, dq, workspace, stream=None):
    _check(_lib.fcp_block_attn_bwd_dq(problem.ref, _ptr(q), _ptr(k), _ptr(v), _ptr(d_o),
                                      _ptr(dq), _ptr(workspace), _stream(stream)))


def fcp_block_attn_bwd_dq_d(problem: Problem, q, k, v, o, lse, d_o, dq, workspace, stream=None):
    _check(_lib.fcp_block_attn_bwd_dq_d(problem.ref, _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(d_o), _ptr(dq),
                                        _ptr(workspace), _stream(stream)))


def fcp_block_attn_bwd_dq_ds(problem: Problem, k, dq, workspace, stream=None):
    _check(_lib.fcp_block_attn_bwd_dq_ds(problem.ref, _ptr(k), _ptr(dq), _ptr(workspace), _stream(stream)))


def fcp_device_info():
    a, b, c = C.c_int32(0), C.c_int32(0), C.c_int32(0)
    _check(_lib.fcp_device_info(C.byref(a), C.byref(b), C.byref(c)))
    return dict(n_compute_units=a.value, fwd_grid=b.value, bwd_grid=c.value)


def fcp_mfma_probe(operand_kind: int, iters: int, out, stream=None):
    """Launches the pure-MFMA measurement kernel; the caller times it.  FLOPs = CUs * 8 * iters * 16 * 32768."""
    _check(_lib.fcp_mfma_probe(int(operand_kind), int(iters), _ptr(out), _stream(stream)))


def fcp_mfma_valu_probe(operand_kind: int, valu_per_mfma: int, iters: int, out, stream=None):
    _check(_lib.fcp_mfma_valu_probe(int(operand_kind), int(valu_per_mfma), int(iters), _ptr(out), _stream(stream)))


def fcp_lds_probe(mode: int, n_waves: int, iters: int, src, out, stream=None):
    _check(_lib.fcp_lds_probe(int(mode), int(n_waves), int(iters), _ptr(src), _ptr(out), _stream(stream)))


def fcp_atomic_probe(buf, n_rows: int, row_stride: int, iters: int, workgroups_per_cu: int, stream=None):
    _check(_lib.fcp_atomic_probe(_ptr(buf), int(n_rows), int(row_stride), int(iters), int(workgroups_per_cu), _stream(stream)))


# ---------------------------------------------------------------- host-side scheduling (fcp_sched.h)
def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def fcp_block_costs(seq_lens, block_size, causal=1):
    """Returns (blocks int32 [n,4], mem int64 [n], comp int64 [n])."""
    sl = _i32(np.asarray(seq_lens).reshape(-1))
    i32p = C.POINTER(C.c_int32)
    n = C.c_int32(0)
    _check(_lib.fcp_block_costs(sl.ctypes.data_as(i32p), len(sl), int(block_size), int(causal), None, None, None, C.byref(n)))
    blocks = np.zeros((max(1, n.value), 4), dtype=np.int32)
    mem = np.zeros(max(1, n.value), dtype=np.int64)
    comp = np.zeros(max(1, n.value), dtype=np.int64)
    _check(_lib.fcp_block_costs(sl.ctypes.data_as(i32p), len(sl), int(block_size), int(causal),
                                blocks.ctypes.data, mem.ctypes.data, comp.ctypes.data, C.byref(n)))
    return blocks[: n.value], mem[: n.value], comp[: n.value]


def fcp_pack_units(blocks, mem, comp, block_size):
    """Returns (unit_of_block int32 [n], unit_mem int64 [U], unit_comp int64 [U])."""
    blocks, mem, comp = _i32(np.asarray(blocks).reshape(-1, 4)), _i64(mem), _i64(comp)
    n = len(mem)
    unit = np.full(max(1, n), -1, dtype=np.int32)
    u_m, u_c = np.zeros(max(1, n), dtype=np.int64), np.zeros(max(1, n), dtype=np.int64)
    cnt = C.c_int32(n)
    _check(_lib.fcp_pack_units(blocks.ctypes.data, mem.ctypes.data, comp.ctypes.data, n, int(block_size),
                               unit.ctypes.data, u_m.ctypes.data, u_c.ctypes.data, C.byref(cnt)))
    return unit[:n], u_m[: cnt.value], u_c[: cnt.value]


def fcp_assign_blocks(mem, comp, n_workers, alpha=1.0, beta=1.0, mem_limit=0, delta=0.0):
    """Returns (owner int32 [n], worker_mem int64 [N], worker_comp int64 [N])."""
    mem, comp = _i64(mem), _i64(comp)
    if mem.shape != comp.shape:
        raise ValueError("mem and comp differ in length")
    owner = np.full(max(1, len(mem)), -1, dtype=np.int32)
    w_m = np.zeros(max(1, int(n_workers)), dtype=np.int64)
    w_c = np.zeros(max(1, int(n_workers)), dtype=np.int64)
    _check(_lib.fcp_assign_blocks(mem.ctypes.data, comp.ctypes.data, len(mem), int(n_workers), float(alpha), float(beta),
                                  int(mem_limit), float(delta), owner.ctypes.data, w_m.ctypes.data, w_c.ctypes.data))
    return owner[: len(mem)], w_m[: max(0, int(n_workers))], w_c[: max(0, int(n_workers))]


def fcp_worker_blocks(blocks, owner, worker):
    """Returns the worker's q_owned table, int32 [n,2] of (seq, idx)."""
    blocks, owner = _i32(np.asarray(blocks).reshape(-1, 4)), _i32(owner)
    n = C.c_int32(0)
    _check(_lib.fcp_worker_blocks(blocks.ctypes.data, owner.ctypes.data, len(owner), int(worker), None, C.byref(n)))
    out = np.zeros((max(1, n.value), 2), dtype=np.int32)
    _check(_lib.fcp_worker_blocks(blocks.ctypes.data, owner.ctypes.data, len(owner), int(worker), out.ctypes.data, C.byref(n)))
    return out[: n.value]


def fcp_comm_edges(blocks, owner, n_workers, causal=1):
    """Returns edges int32 [E,4] of (src, dst, kv_blk, stage = -1)."""
    blocks, owner = _i32(np.asarray(blocks).reshape(-1, 4)), _i32(owner)
    n = C.c_int64(0)
    _check(_lib.fcp_comm_edges(blocks.ctypes.data, owner.ctypes.data, len(owner), int(n_workers), int(causal), None, C.byref(n)))
    edges = np.zeros((max(1, n.value), 4), dtype=np.int32)
    _check(_lib.fcp_comm_edges(blocks.ctypes.data, owner.ctypes.data, len(owner), int(n_workers), int(causal),
                               edges.ctypes.data, C.byref(n)))
    return edges[: n.value]


def fcp_solve_matchings(edges, n_workers):
    """Fills column 3 (sub-stage) of a contiguous int32 [E,4] edge table in place; returns Delta."""
    if not (isinstance(edges, np.ndarray) and edges.dtype == np.int32 and edges.ndim == 2 and edges.shape[1] == 4):
        raise ValueError("edges must be an int32 [E,4] array")
    if len(edges) and not edges.flags["C_CONTIGUOUS"]:
        raise ValueError("edges must be C-contiguous")
    d = C.c_int32(0)
    _check(_lib.fcp_solve_matchings(edges.ctypes.data if len(edges) else None, len(edges), int(n_workers), C.byref(d)))
    return d.value


def fcp_coalesce_stages(edges, coalesce):
    """Returns (stage_of_edge int32 [E], n_stages)."""
    edges = _i32(np.asarray(edges).reshape(-1, 4))
    out = np.zeros(max(1, len(edges)), dtype=np.int32)
    n = C.c_int32(0)
    _check(_lib.fcp_coalesce_stages(edges.ctypes.data if len(edges) else None, len(edges), int(coalesce),
                                    out.ctypes.data if len(edges) else None, C.byref(n)))
    return out[: len(edges)], n.value
