"""Pins for the scheduling oracle: brute force on tiny inputs, closed forms, the textbook
special case of the assignment (plain LPT and its 4/3 bound), a hand-worked example, the
attention oracle's own pair list, and the two lemmas of the congestion-free solver."""
import heapq
import itertools

import numpy as np
import pytest

from oracle import fcp_oracle as orc
from oracle import fcp_sched_oracle as sch


# ------------------------------------------------------------------ block costs
@pytest.mark.parametrize("causal", [1, 0])
def test_block_costs_match_mask_count(causal):
    """c_i counted from the explicit mask matrix of every sequence."""
    seq_lens, bs = [13, 0, 4, 9, 1], 4
    blocks, m, c = sch.block_costs(seq_lens, bs, causal)
    want_m, want_c, want_blocks, row = [], [], [], 0
    for s, L in enumerate(seq_lens):
        mask = np.tril(np.ones((L, L), dtype=np.int64)) if causal else np.ones((L, L), dtype=np.int64)
        for i in range(0, L, bs):
            want_blocks.append((s, i // bs, row + i, min(bs, L - i)))
            want_m.append(min(bs, L - i))
            want_c.append(int(mask[i:i + bs].sum()))
        row += L
    assert blocks.tolist() == [list(b) for b in want_blocks]
    assert m == want_m and c == want_c


def test_block_costs_closed_form_and_zigzag_balance():
    """Causal rows lo..hi-1 attend (hi - lo)(lo + hi + 1) / 2 keys; block i plus block n-1-i of one
    sequence always cost the same (why Zig-Zag pairing balances a sequence)."""
    L, bs = 16 * 96, 96
    _, m, c = sch.block_costs([L], bs, 1)
    n = L // bs
    for i in range(n):
        lo, hi = i * bs, (i + 1) * bs
        assert c[i] == (hi - lo) * (lo + hi + 1) // 2
    pair_cost = {c[i] + c[n - 1 - i] for i in range(n)}
    assert len(pair_cost) == 1
    assert sum(c) == L * (L + 1) // 2


def test_block_costs_agree_with_pair_list():
    """c_i is the unmasked area of the block's (query block, KV block) pairs in the attention oracle's plan."""
    seq_lens, bs = [700, 130, 64, 1000], 128
    blocks, m, c = sch.block_costs(seq_lens, bs, 1)
    for b, blk in enumerate(blocks):
        plan = orc.plan_blocks(seq_lens, bs, 1, 0, q_owned=[(int(blk[0]), int(blk[1]))])
        assert orc.pair_nnz(plan) == c[b]
        assert int(plan["q_blocks"][0][3]) == m[b]


# ------------------------------------------------------------------ assignment
def _plain_lpt(cost, n):
    """Textbook LPT: jobs in descending order, each to the machine that is least loaded."""
    heap = [(0, w) for w in range(n)]
    owner = [-1] * len(cost)
    for i in sorted(range(len(cost)), key=lambda i: -cost[i]):
        load, w = heapq.heappop(heap)
        owner[i] = w
        heapq.heappush(heap, (load + cost[i], w))
    return owner


def test_assign_reduces_to_plain_lpt():
    """With m_i proportional to c_i, alpha = beta and no limit, the two normalised terms are equal and
    the algorithm is LPT on one cost.  Distinct power-of-two-free integer costs avoid ties, whose
    order a heap breaks differently."""
    rng = np.random.default_rng(5)
    for n in (2, 3, 7):
        cost = rng.choice(np.arange(1, 5000), size=40, replace=False).tolist()
        owner, w_m, w_c = sch.assign_blocks(cost, [3 * x for x in cost], n)
        ref = _plain_lpt(cost, n)
        loads = sorted(sum(cost[i] for i in range(40) if ref[i] == w) for w in range(n))
        assert sorted(w_m) == loads
        assert sorted(w_c) == [3 * x for x in loads]


def _brute_opt(cost, n):
    best = None
    for assign in itertools.product(range(n), repeat=len(cost)):
        load = [0] * n
        for i, w in enumerate(assign):
            load[w] += cost[i]
        best = max(load) if best is None else min(best, max(load))
    return best


def test_assign_within_lpt_bound_of_brute_force_optimum():
    """Graham's bound for LPT: makespan <= (4/3 - 1/(3N)) OPT, OPT by exhaustive search."""
    rng = np.random.default_rng(11)
    for n, k in ((2, 9), (3, 8)):
        for _ in range(6):
            cost = rng.integers(1, 50, size=k).tolist()
            _, _, w_c = sch.assign_blocks(cost, cost, n)
            opt = _brute_opt(cost, n)
            assert opt <= max(w_c) <= (4.0 / 3.0 - 1.0 / (3 * n)) * opt + 1e-9


def test_assign_hand_worked_example():
    """Five blocks, two workers, alpha = beta = 1, no limit; worked by hand.
    m = (4,4,2,2,4), c = (10,2,6,1,3): m_hat = 8, c_hat = 11.
    keys max(m/8, c/11) = (.909, .5, .545, .25, .5) -> order 0, 2, 1, 4, 3 (1 before 4: stable).
    b0 -> w0 (tie, lowest index): w0 = (4,10).
    b2: w0 max(6/8, 16/11)=1.45, w1 max(2/8, 6/11)=.545 -> w1 = (2,6).
    b1: w0 max(1, 12/11)=1.09, w1 max(.75, 8/11)=.75 -> w1 = (6,8).
    b4: w0 max(1, 13/11)=1.18, w1 max(10/8, 1)=1.25 -> w0 = (8,13).
    b3: w0 max(10/8, 14/11)=1.27, w1 max(1, 9/11)=1 -> w1 = (8,9)."""
    owner, w_m, w_c = sch.assign_blocks([4, 4, 2, 2, 4], [10, 2, 6, 1, 3], 2)
    assert owner == [0, 1, 1, 1, 0]
    assert w_m == [8, 8] and w_c == [13, 9]


def test_assign_weights_select_the_balanced_resource():
    """beta = 0 leaves only the memory term: the memory loads are those of plain LPT on m, whatever c is."""
    rng = np.random.default_rng(3)
    m = rng.choice(np.arange(1, 3000), size=30, replace=False).tolist()
    c = rng.choice(np.arange(1, 10 ** 6), size=30, replace=False).tolist()
    # the sort key looks at both costs whatever the weights: a compute amount of zero keeps it out of the order
    _, w_m, _ = sch.assign_blocks(m, [0] * 30, 4, alpha=1.0, beta=0.0)
    ref = _plain_lpt(m, 4)
    assert sorted(w_m) == sorted(sum(m[i] for i in range(30) if ref[i] == w) for w in range(4))
    # alpha = 0: compute only
    _, _, w_c = sch.assign_blocks([0] * 30, c, 4, alpha=0.0, beta=1.0)
    ref = _plain_lpt(c, 4)
    assert sorted(w_c) == sorted(sum(c[i] for i in range(30) if ref[i] == w) for w in range(4))


def test_assign_memory_limit():
    """No worker exceeds M (1 + delta); a limit that binds changes the assignment; an impossible one fails."""
    m = [8, 8, 8, 8, 1, 1, 1, 1]
    c = [100, 90, 1, 1, 1, 1, 1, 1]
    free_owner, free_m, _ = sch.assign_blocks(m, c, 2)
    owner, w_m, w_c = sch.assign_blocks(m, c, 2, mem_limit=16, delta=0.25)
    assert max(w_m) <= 16 * 1.25 and sum(w_m) == sum(m) and sum(w_c) == sum(c)
    assert sorted(set(owner)) == [0, 1]
    tight_owner, tight_m, _ = sch.assign_blocks(m, c, 2, mem_limit=18, delta=0.0)
    assert max(tight_m) <= 18
    with pytest.raises(ValueError):
        sch.assign_blocks(m, c, 2, mem_limit=17, delta=0.0)     # 36 tokens cannot fit into 2 x 17


def test_assign_limit_excludes_the_least_loaded_worker():
    """The eligibility test comes before the argmin: a block too big for the lighter worker goes to the other."""
    # order: b0 (m 6), b1 (m 5), b2 (m 5).  b0 -> w0, b1 -> w1; b2: w1 is lighter but 10 > 9 is over the limit.
    owner, w_m, _ = sch.assign_blocks([6, 5, 5], [6, 5, 5], 2, mem_limit=11, delta=0.0)
    assert owner == [0, 1, 1]
    owner, w_m, _ = sch.assign_blocks([6, 5, 5], [6, 5, 5], 2, mem_limit=9, delta=0.25)   # cap 11.25
    assert owner == [0, 1, 1]
    with pytest.raises(ValueError):
        sch.assign_blocks([6, 5, 5], [6, 5, 5], 2, mem_limit=9, delta=0.0)


def test_imbalance_ratio_definition():
    assert sch.imbalance_ratio([10, 10, 10]) == 0.0
    assert sch.imbalance_ratio([10, 5, 0]) == pytest.approx(0.5)
    assert sch.imbalance_ratio([4, 0, 0, 0]) == pytest.approx(0.75)


def test_assignment_balances_lognormal_batches():
    """The paper reports under 5 % compute imbalance for block-level assignment; with 4K blocks and the
    lognormal traces of its appendix the oracle reproduces that band at 8-64 workers."""
    from paper_2605_08524_amd.workloads import length_trace
    for kind in ("lognormal", "bimodal"):
        for n in (8, 64):
            lens = length_trace(kind, n * 131072, seed=1)
            _, m, c = sch.block_costs(lens, 4096, 1)
            _, w_m, w_c = sch.assign_blocks(m, c, n)
            assert sch.imbalance_ratio(w_c) < 0.05, (kind, n, sch.imbalance_ratio(w_c))


# ------------------------------------------------------------------ data flow
@pytest.mark.parametrize("causal", [1, 0])
def test_comm_edges_match_per_worker_pair_lists(causal):
    """For every worker: the remote KV blocks in the attention oracle's pair list of its owned query blocks."""
    rng = np.random.default_rng(9)
    seq_lens, bs, n = [900, 130, 520, 64, 1500], 128, 4
    blocks, m, c = sch.block_costs(seq_lens, bs, causal)
    owner = rng.integers(0, n, size=len(blocks)).tolist()
    edges = sch.comm_edges(blocks, owner, causal)
    assert edges == sorted(edges, key=lambda e: (e[2], e[1]))
    assert len(set(edges)) == len(edges)
    for w in range(n):
        owned = sch.worker_q_owned(blocks, owner, w)
        plan = orc.plan_blocks(seq_lens, bs, causal, 0, q_owned=owned)
        need = {int(p[1]) for p in plan["pairs"]}
        remote = {(owner[kb], w, kb) for kb in need if owner[kb] != w}
        assert remote == {e for e in edges if e[1] == w}


# ------------------------------------------------------------------ congestion-free solver
def _random_multigraph(rng, n, e):
    src = rng.integers(0, n, size=e)
    dst = (src + rng.integers(1, n, size=e)) % n        # no self loops, parallel edges allowed
    return src.tolist(), dst.tolist()


def test_solver_gives_delta_matchings():
    rng = np.random.default_rng(2)
    for n, e in ((2, 5), (3, 10), (5, 40), (8, 100), (16, 300)):
        src, dst = _random_multigraph(rng, n, e)
        stage, delta = sch.solve_matchings(src, dst, n)
        assert delta == sch.check_matchings(src, dst, stage, n)
        assert len(set(stage)) == delta          # a vertex of degree Delta uses every stage


def test_solver_special_graphs():
    n = 6
    # a permutation: one stage
    src, dst = list(range(n)), [(i + 2) % n for i in range(n)]
    stage, delta = sch.solve_matchings(src, dst, n)
    assert delta == 1 and stage == [0] * n
    # one sender to all others: N - 1 stages, one edge each
    src, dst = [0] * (n - 1), list(range(1, n))
    stage, delta = sch.solve_matchings(src, dst, n)
    assert delta == n - 1 and sorted(stage) == list(range(n - 1))
    # all-to-all: N - 1 stages, every one a perfect matching of the N workers
    src = [u for u in range(n) for w in range(n) if u != w]
    dst = [w for u in range(n) for w in range(n) if u != w]
    stage, delta = sch.solve_matchings(src, dst, n)
    assert delta == n - 1
    sch.check_matchings(src, dst, stage, n)
    assert all(stage.count(t) == n for t in range(delta))
    # nothing to send
    assert sch.solve_matchings([], [], n) == ([], 0)


def _min_stages_brute(src, dst, n):
    """Smallest k for which some k-colouring of the edges is congestion-free (exhaustive)."""
    e = len(src)
    for k in range(0, e + 1):
        for col in itertools.product(range(k), repeat=e):
            ok = True
            seen = set()
            for u, w, t in zip(src, dst, col):
                if (0, t, u) in seen or (1, t, w) in seen:
                    ok = False
                    break
                seen.add((0, t, u)); seen.add((1, t, w))
            if ok:
                return k
    return e


def test_delta_is_the_minimum_by_exhaustive_search():
    """Lemma 2 and the construction together: the optimum number of sub-stages equals Delta."""
    rng = np.random.default_rng(4)
    for _ in range(8):
        n = int(rng.integers(2, 5))
        src, dst = _random_multigraph(rng, n, int(rng.integers(1, 7)))
        assert _min_stages_brute(src, dst, n) == sch.max_degree(src, dst, n)
        stage, delta = sch.solve_matchings(src, dst, n)
        assert delta == sch.check_matchings(src, dst, stage, n)


def test_checker_rejects_planted_mistakes():
    src, dst = [0, 0, 1, 2], [1, 2, 2, 0]        # Delta = 2
    good = [0, 1, 0, 1]
    assert sch.check_matchings(src, dst, good, 3) == 2
    with pytest.raises(AssertionError):
        sch.check_matchings(src, dst, [0, 0, 1, 1], 3)      # worker 0 sends twice in stage 0
    with pytest.raises(AssertionError):
        sch.check_matchings(src, dst, [0, 1, 1, 0], 3)      # worker 2 receives twice in stage 1
    with pytest.raises(AssertionError):
        sch.check_matchings(src, dst, [0, 1, 2, 1], 3)      # a third stage
    with pytest.raises(AssertionError):
        sch.check_matchings(src, dst, [0, 1, 0], 3)         # an edge without a stage


def test_coalescer_keeps_per_stage_bounds():
    """After coalescing c sub-stages a worker sends at most c and receives at most c blocks per stage,
    and there are ceil(Delta / c) stages."""
    rng = np.random.default_rng(6)
    n = 8
    src, dst = _random_multigraph(rng, n, 150)
    stage, delta = sch.solve_matchings(src, dst, n)
    for c in (1, 4, 16, 0):
        coarse = sch.coalesce_stages(stage, c)
        n_coarse = max(coarse) + 1
        assert n_coarse == (1 if c <= 0 else -(-delta // c))
        for t in range(n_coarse):
            s = [u for u, k in zip(src, coarse) if k == t]
            r = [w for w, k in zip(dst, coarse) if k == t]
            bound = delta if c <= 0 else c
            assert max(s.count(u) for u in set(s)) <= bound
            assert max(r.count(w) for w in set(r)) <= bound


# ------------------------------------------------------------------ packing of short sequences
def _min_bins_brute(sizes, cap):
    best = len(sizes)
    for assign in itertools.product(range(len(sizes)), repeat=len(sizes)):
        load = {}
        for sz, b in zip(sizes, assign):
            load[b] = load.get(b, 0) + sz
        if max(load.values()) <= cap:
            best = min(best, len(load))
    return best


def test_pack_units_fits_and_is_near_the_minimum():
    """Every unit of short sequences holds at most block_size tokens; first-fit decreasing needs at most
    11/9 OPT + 6/9 units (Dosa's bound), OPT by exhaustive search; long sequences are left alone."""
    rng = np.random.default_rng(8)
    bs = 16
    for _ in range(6):
        short = rng.integers(1, bs, size=6).tolist()
        lens = [40] + short[:3] + [16] + short[3:] + [33]
        blocks, m, c = sch.block_costs(lens, bs, 1)
        unit, um, uc = sch.pack_units(blocks, m, c, bs)
        assert sum(um) == sum(m) and sum(uc) == sum(c)
        n_long = sum(1 for b in blocks if int(lens[int(b[0])]) >= bs)
        sizes = {}
        for i, b in enumerate(blocks):
            if lens[int(b[0])] >= bs:
                assert unit.count(unit[i]) == 1                      # a unit of its own
            else:
                sizes.setdefault(unit[i], []).append(m[i])
        assert all(sum(v) <= bs for v in sizes.values())
        assert len(um) == n_long + len(sizes)
        opt = _min_bins_brute(short, bs)
        assert opt <= len(sizes) <= (11 * opt + 6) // 9
        # units are numbered by their first member
        firsts = [unit.index(u) for u in range(len(um))]
        assert firsts == sorted(firsts)


def test_pack_units_hand_worked():
    """Block size 10, lengths 7, 25, 3, 6, 4, 10 -> blocks of 7 | 10, 10, 5 | 3 | 6 | 4 | 10 tokens.  Short
    sequences: blocks 0 (7), 4 (3), 5 (6), 6 (4); the 5-token tail of the long sequence and the full 10-token
    block are not.  First-fit decreasing: 7 opens A; 6 does not fit A, opens B; 4 fits B (6 + 4); 3 fits A (7 + 3)."""
    blocks, m, c = sch.block_costs([7, 25, 3, 6, 4, 10], 10, 1)
    unit, um, uc = sch.pack_units(blocks, m, c, 10)
    assert m == [7, 10, 10, 5, 3, 6, 4, 10]
    assert unit == [0, 1, 2, 3, 0, 4, 4, 5]
    assert um == [10, 10, 10, 5, 10, 10]
    assert uc[0] == c[0] + c[4] and uc[4] == c[5] + c[6]
