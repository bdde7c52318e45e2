"""The allocation-free forward entry point (fcp_block_attn_fwd_static) against fcp_block_attn_fwd.

Two calls in a row on the same device, the second on a smaller input: the fixed scratch array keeps the
first call's tables, so the second call must not be disturbed by them.  Both entry points run the same
kernel over the same work items; every output row has one writer and a fixed summation order, so the
results are compared bit for bit.  The larger case is also held against the CPU oracle."""
import numpy as np
import pytest
import torch

import paper_2605_08524_amd as fcp
from oracle import fcp_oracle as orc
from paper_2605_08524_amd import workloads
from paper_2605_08524_amd.harness import DevicePath

pytestmark = pytest.mark.gpu


def _both(wl, dev):
    dp = DevicePath(wl, dev, flags=0, backward=False)
    p = dp.problem
    dp.fwd()                                      # fcp_queue_build (in DevicePath) + fcp_block_attn_fwd
    torch.cuda.synchronize(dev)
    want_o = dp.o_part[: p.n_slot_rows].clone()
    want_l = dp.lse_part[: p.n_slot_rows].clone()
    dp.o_part.fill_(float("nan"))
    dp.lse_part.fill_(float("nan"))
    torch.cuda.synchronize(dev)
    before = torch.cuda.memory_allocated(dev)
    fcp.fcp_block_attn_fwd_static(p, dp.q, dp.k, dp.v, dp.o_part, dp.lse_part, None)
    torch.cuda.synchronize(dev)
    assert torch.cuda.memory_allocated(dev) == before
    got_o = dp.o_part[: p.n_slot_rows]
    got_l = dp.lse_part[: p.n_slot_rows]
    assert torch.equal(got_o.view(torch.int32), want_o.view(torch.int32)), f"{wl.name}: o_part differs"
    assert torch.equal(got_l.view(torch.int32), want_l.view(torch.int32)), f"{wl.name}: lse_part differs"
    return dp, got_o.float().cpu().numpy(), got_l.cpu().numpy()


def test_static_forward_equals_workspace_forward_twice_in_a_row():
    dev = torch.device("cuda:0")
    big = workloads.custom_workload([1500, 300, 77, 2049], 256, causal=1, coalesce=2, n_q_heads=8, n_kv_heads=2,
                                    head_dim=128, seed=41, name="static-first")
    small = workloads.custom_workload([129, 40], 128, causal=1, coalesce=1, n_q_heads=4, n_kv_heads=4,
                                      head_dim=64, seed=42, name="static-second-smaller")
    print(f"case {big.name} then {small.name}", flush=True)
    for wl in (big, small):
        dp, o_part, lse_part = _both(wl, dev)
        plan = orc.plan_blocks(wl.seq_lens, wl.block_size, wl.causal, wl.coalesce)
        op, lp = orc.partial_fwd(wl.q(), wl.k(), wl.v(), plan, wl.block_size, wl.causal)
        assert np.max(np.abs(o_part - op)) <= 2e-2
        fin = np.isfinite(lp)
        assert np.array_equal(np.isneginf(lse_part), np.isneginf(lp)) and np.max(np.abs(lse_part[fin] - lp[fin])) <= 1e-3
        del dp


def test_static_forward_rejects_what_does_not_fit():
    dev = torch.device("cuda:0")
    wl = workloads.custom_workload([300], 128, causal=1, coalesce=0, n_q_heads=4, n_kv_heads=4, head_dim=64, seed=1, name="static-direct")
    dp = DevicePath(wl, dev, flags=fcp.FCP_FLAG_DIRECT_SINGLE, backward=False)
    with pytest.raises(fcp.FcpError) as e:
        fcp.fcp_block_attn_fwd_static(dp.problem, dp.q, dp.k, dp.v, dp.o_part, dp.lse_part, None)
    assert e.value.code == fcp.binding.FCP_ERR_INVALID_ARG
    # more forward items than the fixed array holds: tables only, no tensor is touched before the size check
    lens = np.full(64, 4096, dtype=np.int32)
    plan = fcp.fcp_plan_blocks(lens, 128, 1, 1)
    prob = fcp.Problem(plan, 32, 8, 128, 128)
    with pytest.raises(fcp.FcpError) as e:
        fcp.fcp_block_attn_fwd_static(prob, dp.q, dp.k, dp.v, dp.o_part, dp.lse_part, None)
    assert e.value.code == fcp.binding.FCP_ERR_BUFFER_TOO_SMALL
