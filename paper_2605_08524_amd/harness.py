"""Device-side plumbing shared by the tests, the smoke check and the benchmark: uploads a
workload's tensors with PyTorch, allocates outputs and the workspace, and calls the C ABI.
No arithmetic of the method happens here."""
from __future__ import annotations

import time

import numpy as np
import torch

from . import binding as B


def to_dev_bf16(bits: np.ndarray, device) -> torch.Tensor:
    """uint16 bf16 bit patterns -> torch.bfloat16 tensor on `device` (bit-exact)."""
    t = torch.from_numpy(bits.view(np.int16)).to(device)
    return t.view(torch.bfloat16)


def packed_plan(wl):
    """The workload's plan with its short sequences packed into shared blocks: block costs -> scheduling units ->
    fcp_plan_blocks_packed, all in the library's host code."""
    blocks, mem, comp = B.fcp_block_costs(wl.seq_lens, wl.block_size, wl.causal)
    unit_of_block = B.fcp_pack_units(blocks, mem, comp, wl.block_size)[0] if len(blocks) else None
    return B.fcp_plan_blocks_packed(wl.seq_lens, wl.block_size, wl.causal, wl.coalesce, wl.q_owned, unit_of_block)


def buffer_rows(wl, plan):
    """Where the rows of a plan's buffers come from in the workload's tensors, which are sequence-major (K / V: all
    tokens by sequence; Q / dO: the owned blocks by (seq, idx)).  Returns (kv_src, q_src), int64 index arrays; for a
    plan without packed blocks both are the identity.  Pure table look-ups: the plan fixes the layout."""
    bs = wl.block_size
    seq_off = np.concatenate([[0], np.cumsum(np.asarray(wl.seq_lens, dtype=np.int64))])
    flat = B.fcp_plan_blocks(wl.seq_lens, bs, wl.causal, 0, wl.q_owned)["q_blocks"]
    q_home = {(int(s), int(i)): int(st) for s, i, st, _ in flat}          # (seq, idx) -> first row in the workload's Q
    members = {}
    for kb, s, off, ln in plan.get("segments", ()):
        members.setdefault(int(kb), []).append((int(s), int(ln)))
    kv_index = {(int(b[0]), int(b[1])): n for n, b in enumerate(plan["kv_blocks"])}
    kv_src, q_src = [], []
    for kb, (s, i, _, ln) in enumerate(plan["kv_blocks"]):
        if kb in members:
            kv_src += [seq_off[ms] + np.arange(mlen) for ms, mlen in members[kb]]
        else:
            kv_src.append(seq_off[s] + int(i) * bs + np.arange(ln))
    for s, i, _, ln in plan["q_blocks"]:
        kb = kv_index[(int(s), int(i))]
        if kb in members:
            q_src += [q_home[(ms, 0)] + np.arange(mlen) for ms, mlen in members[kb]]
        else:
            q_src.append(q_home[(int(s), int(i))] + np.arange(ln))
    cat = lambda parts: np.concatenate(parts).astype(np.int64) if parts else np.zeros(0, dtype=np.int64)
    return cat(kv_src), cat(q_src)


class DevicePath:
    """Holds the device buffers of one workload and runs the path's calls on them.  packed=True plans the workload
    with fcp_plan_blocks_packed and lays the tensors out in that plan's order (kv_src / q_src say which row of the
    workload's sequence-major tensors each buffer row holds)."""

    def __init__(self, wl, device, flags=0, backward=False, stream=None, softmax_scale=0.0, packed=False):
        self.wl, self.device, self.stream = wl, device, stream
        t0 = time.perf_counter()
        if packed:
            self.plan = packed_plan(wl)
        else:
            self.plan = B.fcp_plan_blocks(wl.seq_lens, wl.block_size, wl.causal, wl.coalesce, wl.q_owned)
        self.plan_ms = (time.perf_counter() - t0) * 1e3              # host: block table, pair list, slots
        self.problem = B.Problem(self.plan, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.block_size, softmax_scale, flags)
        p = self.problem
        Hq, Hkv, d = wl.n_q_heads, wl.n_kv_heads, wl.head_dim
        self.kv_src, self.q_src = buffer_rows(wl, self.plan) if packed else (None, None)
        lay_q = (lambda x: x[self.q_src]) if packed else (lambda x: x)
        lay_kv = (lambda x: x[self.kv_src]) if packed else (lambda x: x)
        self.q = to_dev_bf16(lay_q(wl.q()), device)
        self.k = to_dev_bf16(lay_kv(wl.k()), device)
        self.v = to_dev_bf16(lay_kv(wl.v()), device)
        f32 = dict(dtype=torch.float32, device=device)
        nan = float("nan")
        part_dtype = torch.bfloat16 if (flags & B.FCP_FLAG_PART_BF16) else torch.float32
        self.o_part = torch.full((max(1, p.n_slot_rows), Hq, d), nan, dtype=part_dtype, device=device)
        self.lse_part = torch.full((max(1, p.n_slot_rows), Hq), nan, **f32)
        o_dtype = torch.float32 if (flags & B.FCP_FLAG_O_F32) else torch.bfloat16
        self.o = torch.full((max(1, p.t_q), Hq, d), nan, dtype=o_dtype, device=device)
        self.lse = torch.full((max(1, p.t_q), Hq), nan, **f32)
        self.ws_bytes = B.fcp_workspace_bytes(p)
        self.ws = torch.empty(self.ws_bytes + 256, dtype=torch.uint8, device=device)
        self.ws.fill_(0xFF)      # poison (bf16 / fp32 NaN patterns): whatever a kernel reads must have been written first
        off = (-self.ws.data_ptr()) % 256
        self.ws_ptr = self.ws.data_ptr() + off
        torch.cuda.synchronize(device)
        t0 = time.perf_counter()
        B.fcp_queue_build(p, self.ws_ptr, self.ws_bytes, stream)
        self.queue_build_ms = (time.perf_counter() - t0) * 1e3     # host: work items + one upload (returns when it is done)
        if backward:
            self.d_o = to_dev_bf16(lay_q(wl.d_o()), device)
            g_dtype = torch.bfloat16 if (flags & B.FCP_FLAG_GRAD_BF16) else torch.float32
            self.dq = torch.full((max(1, p.t_q), Hq, d), nan, dtype=g_dtype, device=device)
            self.dk = torch.full((max(1, p.t_kv), Hkv, d), nan, dtype=g_dtype, device=device)
            self.dv = torch.full((max(1, p.t_kv), Hkv, d), nan, dtype=g_dtype, device=device)

    def fwd(self):
        if self.problem.flags & B.FCP_FLAG_DIRECT_SINGLE:
            B.fcp_block_attn_fwd_out(self.problem, self.q, self.k, self.v, self.o_part, self.lse_part,
                                     self.o, self.lse, self.ws_ptr, self.stream)
        else:
            B.fcp_block_attn_fwd(self.problem, self.q, self.k, self.v, self.o_part, self.lse_part, self.ws_ptr, self.stream)

    def merge(self):
        B.fcp_merge_partials(self.problem, self.o_part, self.lse_part, self.o, self.lse, self.ws_ptr, self.stream)

    def bwd(self):
        B.fcp_block_attn_bwd(self.problem, self.q, self.k, self.v, self.o, self.lse, self.d_o,
                             self.dq, self.dk, self.dv, self.ws_ptr, self.stream)


    def bwd_pre(self):
        B.fcp_bwd_preprocess(self.problem, self.o, self.lse, self.d_o, self.ws_ptr, self.stream)

    def bwd_dq_d(self):
        B.fcp_block_attn_bwd_dq_d(self.problem, self.q, self.k, self.v, self.o, self.lse, self.d_o,
                                  self.dq, self.ws_ptr, self.stream)

    def bwd_dkdv(self):
        B.fcp_block_attn_bwd_dkdv(self.problem, self.q, self.k, self.v, self.d_o,
                                  self.dk, self.dv, self.ws_ptr, self.stream)

    def bwd_dq_ds(self):
        B.fcp_block_attn_bwd_dq_ds(self.problem, self.k, self.dq, self.ws_ptr, self.stream)

    def bwd_dq(self):
        B.fcp_block_attn_bwd_dq(self.problem, self.q, self.k, self.v, self.d_o,
                                self.dq, self.ws_ptr, self.stream)


def run_path(wl, device, backward=False, flags=0, softmax_scale=0.0, packed=False):
    """One pass of the whole path; returns host copies (numpy) of every output, in the layout of the plan's buffers."""
    dp = DevicePath(wl, device, flags=flags, backward=backward, softmax_scale=softmax_scale, packed=packed)
    dp.fwd()
    dp.merge()
    if backward:
        dp.bwd()
    torch.cuda.synchronize(device)
    p = dp.problem
    out = dict(plan=dp.plan, o_part=dp.o_part[: p.n_slot_rows].float().cpu().numpy(),
               lse_part=dp.lse_part[: p.n_slot_rows].cpu().numpy(),
               o=dp.o[: p.t_q].float().cpu().numpy(), lse=dp.lse[: p.t_q].cpu().numpy())
    if backward:
        out.update(dq=dp.dq[: p.t_q].float().cpu().numpy(), dk=dp.dk[: p.t_kv].float().cpu().numpy(),
                   dv=dp.dv[: p.t_kv].float().cpu().numpy())
    return out


class RunningPath:
    """The forward as a loop over execution stages with a running result (FCP_FLAG_RUNNING_MERGE): stage k = the k-th
    slot of every query block; each stage is one fcp_block_attn_fwd_out launch that folds its slots into (o, lse) in
    place.  No partial buffers exist.  The stages' tables and work queues are built once, up front."""

    def __init__(self, wl, device, softmax_scale=0.0, stream=None):
        self.wl, self.device, self.stream = wl, device, stream
        self.plan = B.fcp_plan_blocks(wl.seq_lens, wl.block_size, wl.causal, wl.coalesce, wl.q_owned)
        _, self.n_stages = B.fcp_stage_tables(self.plan, 0)
        self.q, self.k, self.v = (to_dev_bf16(x, device) for x in (wl.q(), wl.k(), wl.v()))
        self.t_q = int(self.plan["q_blocks"][:, 3].sum()) if len(self.plan["q_blocks"]) else 0
        self.o = torch.full((max(1, self.t_q), wl.n_q_heads, wl.head_dim), float("nan"), dtype=torch.float32, device=device)
        self.lse = torch.empty((max(1, self.t_q), wl.n_q_heads), dtype=torch.float32, device=device)
        self.stages = []
        for st in range(self.n_stages):
            sp, _ = B.fcp_stage_tables(self.plan, st)
            prob = B.Problem(sp, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.block_size, softmax_scale,
                             B.FCP_FLAG_RUNNING_MERGE | B.FCP_FLAG_O_F32)
            nbytes = B.fcp_workspace_bytes(prob)
            ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
            ws_ptr = ws.data_ptr() + (-ws.data_ptr()) % 256
            B.fcp_queue_build(prob, ws_ptr, nbytes, stream)
            self.stages.append((prob, ws, ws_ptr))

    def fwd(self):
        self.lse.fill_(float("-inf"))        # "nothing yet": the first stage of every row then ignores what o holds
        for prob, _, ws_ptr in self.stages:
            B.fcp_block_attn_fwd_out(prob, self.q, self.k, self.v, None, None, self.o, self.lse, ws_ptr, self.stream)


def run_running_forward(wl, device, softmax_scale=0.0, stream=None):
    """One pass of the staged forward with a running result; returns host copies of o and lse, the plan and the
    number of stages."""
    rp = RunningPath(wl, device, softmax_scale, stream)
    rp.fwd()
    torch.cuda.synchronize(device)
    return dict(o=rp.o[:rp.t_q].cpu().numpy(), lse=rp.lse[:rp.t_q].cpu().numpy(), plan=rp.plan, n_stages=rp.n_stages)
