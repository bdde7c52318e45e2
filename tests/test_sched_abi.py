"""The host-side scheduling of the C-ABI library against the scheduling oracle: block costs, owners and
data-flow edges bit for bit; the congestion-free ordering on what is unique (the number of sub-stages)
and by the oracle's validity check for the rest."""
import numpy as np
import pytest

import paper_2605_08524_amd as fcp
from oracle import fcp_oracle as orc
from oracle import fcp_sched_oracle as sch
from paper_2605_08524_amd import workloads


def _traces():
    yield "tiny", [13, 0, 4, 9, 1], 4
    yield "ragged", [700, 130, 64, 1000, 1, 128, 129], 128
    yield "lognormal", workloads.length_trace("lognormal", 8 * 131072, seed=0), 4096
    yield "bimodal", workloads.length_trace("bimodal", 16 * 131072, seed=2), 4096


TRACES = list(_traces())


@pytest.mark.parametrize("name,lens,bs", TRACES, ids=[t[0] for t in TRACES])
@pytest.mark.parametrize("causal", [1, 0])
def test_block_costs_match_oracle(name, lens, bs, causal):
    blocks, mem, comp = fcp.fcp_block_costs(lens, bs, causal)
    ref_blocks, ref_m, ref_c = sch.block_costs(lens, bs, causal)
    assert blocks.dtype == np.int32 and mem.dtype == np.int64 and comp.dtype == np.int64
    assert np.array_equal(blocks, ref_blocks)
    assert mem.tolist() == ref_m and comp.tolist() == ref_c


def test_block_costs_agree_with_the_planner_tables():
    """Same blocks as fcp_plan_blocks produces for a worker that owns everything."""
    lens, bs = [700, 130, 64, 1000, 1, 128, 129], 128
    blocks, mem, comp = fcp.fcp_block_costs(lens, bs, 1)
    plan = fcp.fcp_plan_blocks(lens, bs, 1, 0)
    assert np.array_equal(blocks, plan["kv_blocks"])


@pytest.mark.parametrize("name,lens,bs", TRACES, ids=[t[0] for t in TRACES])
@pytest.mark.parametrize("n_workers", [1, 3, 8, 64])
@pytest.mark.parametrize("alpha,beta", [(1.0, 1.0), (0.3, 1.0), (1.0, 0.0)])
def test_assignment_matches_oracle(name, lens, bs, n_workers, alpha, beta):
    _, m, c = sch.block_costs(lens, bs, 1)
    ref_owner, ref_m, ref_c = sch.assign_blocks(m, c, n_workers, alpha, beta)
    owner, w_m, w_c = fcp.fcp_assign_blocks(m, c, n_workers, alpha, beta)
    assert owner.tolist() == ref_owner
    assert w_m.tolist() == ref_m and w_c.tolist() == ref_c


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_assignment_with_memory_limit_matches_oracle(seed):
    rng = np.random.default_rng(seed)
    lens = workloads.length_trace("lognormal", 8 * 65536, seed=seed)
    _, m, c = sch.block_costs(lens, 2048, 1)
    n = 8
    # a limit that binds: 2 % above the average load, plus a tolerance
    limit = int(sum(m) / n * 1.02)
    for delta in (0.0, 0.05):
        try:
            ref = sch.assign_blocks(m, c, n, 1.0, 1.0, limit, delta)
        except ValueError:
            with pytest.raises(fcp.FcpError) as err:
                fcp.fcp_assign_blocks(m, c, n, 1.0, 1.0, limit, delta)
            assert err.value.code == fcp.FCP_ERR_INFEASIBLE
            continue
        owner, w_m, w_c = fcp.fcp_assign_blocks(m, c, n, 1.0, 1.0, limit, delta)
        assert owner.tolist() == ref[0] and w_m.tolist() == ref[1] and w_c.tolist() == ref[2]
        assert max(w_m) <= limit * (1 + delta)
    # random small integer costs: many equal keys and equal loads, so the tie rules decide
    m2 = rng.integers(1, 4, size=200).tolist()
    c2 = rng.integers(0, 3, size=200).tolist()
    ref = sch.assign_blocks(m2, c2, 7, 1.0, 1.0, 70, 0.0)
    owner, w_m, w_c = fcp.fcp_assign_blocks(m2, c2, 7, 1.0, 1.0, 70, 0.0)
    assert owner.tolist() == ref[0] and w_m.tolist() == ref[1] and w_c.tolist() == ref[2]


def test_assignment_errors():
    with pytest.raises(fcp.FcpError) as err:
        fcp.fcp_assign_blocks([6, 5, 5], [6, 5, 5], 2, mem_limit=9)
    assert err.value.code == fcp.FCP_ERR_INFEASIBLE
    for bad in (dict(n_workers=0), dict(n_workers=2, alpha=-1.0), dict(n_workers=2, delta=float("nan"))):
        with pytest.raises(fcp.FcpError) as err:
            fcp.fcp_assign_blocks([1, 2], [1, 2], **bad)
        assert err.value.code == -1
    with pytest.raises(fcp.FcpError):
        fcp.fcp_assign_blocks([1, -2], [1, 2], 2)
    owner, w_m, w_c = fcp.fcp_assign_blocks([], [], 3)
    assert len(owner) == 0 and w_m.tolist() == [0, 0, 0]


@pytest.mark.parametrize("name,lens,bs", TRACES, ids=[t[0] for t in TRACES])
@pytest.mark.parametrize("causal", [1, 0])
def test_edges_and_worker_tables_match_oracle(name, lens, bs, causal):
    n = 8
    blocks, m, c = sch.block_costs(lens, bs, causal)
    owner, _, _ = sch.assign_blocks(m, c, n)
    ref = sch.comm_edges(blocks, owner, causal)
    edges = fcp.fcp_comm_edges(blocks, owner, n, causal)
    assert edges.shape == (len(ref), 4)
    assert [tuple(e[:3]) for e in edges.tolist()] == ref
    assert (edges[:, 3] == -1).all()
    for w in range(n):
        assert [tuple(r) for r in fcp.fcp_worker_blocks(blocks, owner, w).tolist()] == sch.worker_q_owned(blocks, owner, w)


def test_edges_reject_bad_tables():
    blocks, m, c = sch.block_costs([10, 10], 4, 1)
    with pytest.raises(fcp.FcpError):
        fcp.fcp_comm_edges(blocks, [0, 1, 2, 0, 1, 9], 3, 1)            # owner out of range
    with pytest.raises(fcp.FcpError):
        fcp.fcp_comm_edges(blocks[::-1].copy(), [0, 1, 2, 0, 1, 2], 3, 1)  # not in (seq, idx) order


def _random_multigraph(rng, n, e):
    src = rng.integers(0, n, size=e)
    dst = (src + rng.integers(1, n, size=e)) % n
    return np.stack([src, dst, np.zeros(e, dtype=np.int64), np.full(e, -1)], axis=1).astype(np.int32)


@pytest.mark.parametrize("n,e", [(2, 1), (2, 7), (3, 10), (5, 40), (8, 100), (16, 1000), (64, 5000), (256, 20000)])
def test_solver_uses_delta_valid_substages(n, e):
    rng = np.random.default_rng(n * 1000 + e)
    edges = _random_multigraph(rng, n, e)
    before = edges[:, :3].copy()
    delta = fcp.fcp_solve_matchings(edges, n)
    assert np.array_equal(edges[:, :3], before)                  # the edge multiset is untouched
    assert delta == sch.check_matchings(edges[:, 0].tolist(), edges[:, 1].tolist(), edges[:, 3].tolist(), n)
    assert delta == sch.solve_matchings(edges[:, 0].tolist(), edges[:, 1].tolist(), n)[1]


def test_solver_on_assigned_batches():
    """The whole host chain on the appendix traces: costs -> owners -> edges -> sub-stages -> stages."""
    for kind, n in (("lognormal", 8), ("bimodal", 32)):
        lens = workloads.length_trace(kind, n * 131072, seed=3)
        blocks, mem, comp = fcp.fcp_block_costs(lens, 4096, 1)
        owner, w_m, w_c = fcp.fcp_assign_blocks(mem, comp, n)
        edges = fcp.fcp_comm_edges(blocks, owner, n, 1)
        delta = fcp.fcp_solve_matchings(edges, n)
        assert delta == sch.check_matchings(edges[:, 0].tolist(), edges[:, 1].tolist(), edges[:, 3].tolist(), n)
        for c in (1, 4, 16, 0):
            stage, n_stages = fcp.fcp_coalesce_stages(edges, c)
            assert stage.tolist() == sch.coalesce_stages(edges[:, 3].tolist(), c)
            assert n_stages == (1 if c == 0 else -(-delta // c))
            bound = delta if c == 0 else c
            for t in range(n_stages):
                sel = edges[stage == t]
                assert np.bincount(sel[:, 0], minlength=n).max() <= bound
                assert np.bincount(sel[:, 1], minlength=n).max() <= bound


def test_solver_special_graphs_and_errors():
    n = 6
    perm = np.array([[i, (i + 2) % n, 0, -1] for i in range(n)], dtype=np.int32)
    assert fcp.fcp_solve_matchings(perm, n) == 1 and (perm[:, 3] == 0).all()
    star = np.array([[0, w, 0, -1] for w in range(1, n)], dtype=np.int32)
    assert fcp.fcp_solve_matchings(star, n) == n - 1 and sorted(star[:, 3].tolist()) == list(range(n - 1))
    full = np.array([[u, w, 0, -1] for u in range(n) for w in range(n) if u != w], dtype=np.int32)
    assert fcp.fcp_solve_matchings(full, n) == n - 1
    sch.check_matchings(full[:, 0].tolist(), full[:, 1].tolist(), full[:, 3].tolist(), n)
    assert fcp.fcp_solve_matchings(np.zeros((0, 4), dtype=np.int32), n) == 0
    bad = np.array([[0, 7, 0, -1]], dtype=np.int32)
    with pytest.raises(fcp.FcpError):
        fcp.fcp_solve_matchings(bad, n)
    with pytest.raises(fcp.FcpError):
        fcp.fcp_coalesce_stages(np.array([[0, 1, 0, -1]], dtype=np.int32), 4)     # no sub-stage yet


def test_worker_share_feeds_the_planner():
    """A worker's block list from the assignment is a valid q_owned table: the planner accepts it and its pair
    list names exactly the worker's remote blocks plus its local ones."""
    lens, bs, n = workloads.length_trace("lognormal", 4 * 32768, seed=5), 1024, 4
    blocks, mem, comp = fcp.fcp_block_costs(lens, bs, 1)
    owner, _, _ = fcp.fcp_assign_blocks(mem, comp, n)
    edges = fcp.fcp_comm_edges(blocks, owner, n, 1)
    for w in range(n):
        q_owned = fcp.fcp_worker_blocks(blocks, owner, w)
        plan = fcp.fcp_plan_blocks(lens, bs, 1, 16, q_owned)
        ref = orc.plan_blocks(lens, bs, 1, 16, q_owned=[tuple(r) for r in q_owned.tolist()])
        assert np.array_equal(plan["pairs"], np.asarray(ref["pairs"], dtype=np.int32).reshape(-1, 4))
        need = set(plan["pairs"][:, 1].tolist())
        assert {kb for kb in need if owner[kb] != w} == set(edges[edges[:, 1] == w][:, 2].tolist())


def test_pack_units_matches_oracle():
    rng = np.random.default_rng(12)
    cases = [([7, 25, 3, 6, 4, 10], 10), ([13, 0, 4, 9, 1], 4), ([5], 8), ([], 8)]
    for _ in range(6):
        lens = np.where(rng.random(60) < 0.7, rng.integers(1, 1024, size=60), rng.integers(1024, 9000, size=60))
        cases.append((lens.tolist(), 1024))
    for lens, bs in cases:
        blocks, m, c = sch.block_costs(lens, bs, 1)
        ref = sch.pack_units(blocks, m, c, bs)
        unit, u_m, u_c = fcp.fcp_pack_units(blocks, m, c, bs)
        assert unit.tolist() == ref[0] and u_m.tolist() == ref[1] and u_c.tolist() == ref[2]


def test_units_flow_through_assignment_and_planner():
    """Short sequences assigned as shared units: every member of a unit lands on the same worker, and the
    worker tables built from it are what the planner accepts."""
    rng = np.random.default_rng(13)
    lens = np.where(rng.random(80) < 0.75, rng.integers(16, 512, size=80), rng.integers(2000, 12000, size=80))
    bs, n = 1024, 4
    blocks, mem, comp = fcp.fcp_block_costs(lens, bs, 1)
    unit, u_m, u_c = fcp.fcp_pack_units(blocks, mem, comp, bs)
    assert len(u_m) < len(mem) and u_m[np.bincount(unit) > 1].max() <= bs
    u_owner, w_m, w_c = fcp.fcp_assign_blocks(u_m, u_c, n)
    owner = u_owner[unit]
    assert w_m.sum() == mem.sum() and np.array_equal(np.bincount(owner, weights=mem, minlength=n).astype(np.int64), w_m)
    for w in range(n):
        q_owned = fcp.fcp_worker_blocks(blocks, owner, w)
        plan = fcp.fcp_plan_blocks(lens, bs, 1, 16, q_owned)
        assert int(plan["q_blocks"][:, 3].sum()) == int(w_m[w])
