"""CPU oracle for the host-side scheduling of FCP: block costs, the greedy load-balanced
assignment, the data-flow graph and its congestion-free ordering, the coalescer.

TEST INFRASTRUCTURE ONLY.  Plain Python / numpy, integers as Python ints, loads in
IEEE double.  Only the tests and the benchmark's CPU-baseline leg may import it; it
imports nothing from the product package and shares no code with the C++ library.

What it follows (all from the paper):

* Block costs (appendix "Block Assignment Algorithm", first paragraph): every block i
  has a memory usage m_i and a compute amount c_i.  Read here as m_i = tokens of the
  block, c_i = number of unmasked (query row, key column) score entries of the block's
  query rows, per head; the paper gives no formula (it only says that both are estimated
  from the length of the sequence the block comes from).
* Short sequences (section "Block Distributor", sharding policy) are packed into shared units by
  first-fit decreasing; the paper asks for as few blocks as possible and names no rule.
* Greedy Load-Balanced Assignment (appendix algorithm of that name): average loads,
  descending sort by max(m_i / m_hat, c_i / c_hat), then every block goes to the
  eligible worker with the smallest max(alpha (m_w + m_i) / m_hat, beta (c_w + c_i) / c_hat).
  Readings where the listing is silent: the sort is stable (equal keys keep block
  order); among equal loads the lowest worker index wins; mem_limit <= 0 means no
  limit; if no worker is eligible for a block the assignment fails (ValueError).
* Imbalance ratio (section "Workload Balance" of the evaluation): (max - mean) / max.
* Data-flow graph (section "Communication Planner", congestion-free solver, and the
  caption of its figure): one edge S(u) -> R(w) for every KV block owned by u that a
  query block owned by w != u depends on; a worker pulls a block once however many of
  its query blocks need it.
* Congestion-free solver (same section, Lemmas 1 and 2, appendix "Proof of
  Congestion-Free Solver"): the edges are split into exactly Delta matchings
  (Delta = maximum degree) by padding the graph to Delta-regular and removing one
  perfect matching after another.  The matchings themselves are not unique; what is
  unique is their number, and `check_matchings` states what makes a split valid.
* Bottom-up coalescer (same section): c consecutive sub-stages form one stage.

Pinned by tests/test_sched_oracle_pins.py.
"""
from __future__ import annotations

import numpy as np
from scipy.sparse import csr_matrix
from scipy.sparse.csgraph import maximum_bipartite_matching


# --------------------------------------------------------------------------
# blocks and their costs
# --------------------------------------------------------------------------
def block_costs(seq_lens, block_size, causal=1):
    """Blocks of every sequence, by (seq, idx), with m_i and c_i.

    Returns (blocks [n,4] = (seq, idx, tok_start, tok_len), m [n], c [n]) with m, c as
    Python-int lists.  tok_start is the row in the packed token buffer.  c_i counts, for
    every query row of the block (position p in its sequence of length L), the keys it
    attends: p + 1 under a causal mask, L otherwise.
    """
    blocks, m, c = [], [], []
    row = 0
    for s, L in enumerate(seq_lens):
        L = int(L)
        n = (L + block_size - 1) // block_size
        for i in range(n):
            lo = i * block_size
            hi = min(L, lo + block_size)
            blocks.append((s, i, row + lo, hi - lo))
            m.append(hi - lo)
            if causal:
                c.append(sum(p + 1 for p in range(lo, hi)))
            else:
                c.append((hi - lo) * L)
        row += L
    return np.asarray(blocks, dtype=np.int64).reshape(-1, 4), m, c


# --------------------------------------------------------------------------
# packing of short sequences into scheduling units
# --------------------------------------------------------------------------
def pack_units(blocks, m, c, block_size):
    """Scheduling units: a sequence shorter than a block does not get a block of its own but shares one with
    other short sequences (section "Block Distributor", sharding policy: short sequences are packed into as
    few blocks as possible and run through the variable-length path).  The paper names no packing rule;
    read here as first-fit decreasing: the short sequences in descending length (equal lengths in block
    order) each go into the first open unit with room, else open a new one.  Every block of a sequence that
    has at least block_size tokens is a unit by itself.  Units are numbered by their first member block.
    Returns (unit_of_block [K], unit_m [U], unit_c [U])."""
    K = len(m)
    n_in_seq = {}
    for b in blocks:
        n_in_seq[int(b[0])] = n_in_seq.get(int(b[0]), 0) + 1
    short = [i for i in range(K) if n_in_seq[int(blocks[i][0])] == 1 and m[i] < block_size]
    bins = []                     # [free tokens, member list]
    for i in sorted(short, key=lambda i: -m[i]):
        for bn in bins:
            if bn[0] >= m[i]:
                bn[0] -= m[i]
                bn[1].append(i)
                break
        else:
            bins.append([block_size - m[i], [i]])
    groups = [[i] for i in range(K) if i not in set(short)] + [sorted(bn[1]) for bn in bins]
    groups.sort(key=lambda g: g[0])
    unit_of_block = [-1] * K
    for u, g in enumerate(groups):
        for i in g:
            unit_of_block[i] = u
    return unit_of_block, [sum(m[i] for i in g) for g in groups], [sum(c[i] for i in g) for g in groups]


# --------------------------------------------------------------------------
# Greedy Load-Balanced Assignment
# --------------------------------------------------------------------------
def assign_blocks(m, c, n_workers, alpha=1.0, beta=1.0, mem_limit=0, delta=0.0):
    """Greedy assignment of blocks to workers (appendix "Block Assignment Algorithm").

    Every worker should end up with the batch's mean memory and mean compute; a block's size is the
    larger of its memory and compute cost relative to those means; blocks are placed largest first,
    each on the worker that would be least loaded afterwards (load = the larger of its weighted
    relative memory and compute), among the workers whose memory stays within mem_limit * (1 + delta).
    Returns (owner [K], worker_m [N], worker_c [N])."""
    K, N = len(m), int(n_workers)
    if N <= 0:
        raise ValueError("no workers")
    m = [int(x) for x in m]
    c = [int(x) for x in c]
    # mean cost per worker (the sums are exact integers)
    m_hat = float(sum(m)) / N
    c_hat = float(sum(c)) / N
    # a cost that is zero for every block drops out of both the key and the load
    def rel(x, x_hat):
        return float(x) / x_hat if x_hat > 0.0 else 0.0
    # largest relative cost first; equal keys keep their block order
    key = [max(rel(m[i], m_hat), rel(c[i], c_hat)) for i in range(K)]
    order = sorted(range(K), key=lambda i: -key[i])
    w_m, w_c = [0] * N, [0] * N
    owner = [-1] * K
    cap = float(mem_limit) * (1.0 + float(delta))
    # ties between workers go to the lowest index
    for i in order:
        best, best_load = -1, 0.0
        for w in range(N):
            if mem_limit > 0 and float(w_m[w] + m[i]) > cap:
                continue
            load = max(alpha * rel(w_m[w] + m[i], m_hat), beta * rel(w_c[w] + c[i], c_hat))
            if best < 0 or load < best_load:
                best, best_load = w, load
        if best < 0:
            raise ValueError(f"block {i} fits on no worker")
        owner[i] = best
        w_m[best] += m[i]
        w_c[best] += c[i]
    return owner, w_m, w_c


def imbalance_ratio(load):
    """(max - mean) / max of the per-worker loads; 0 for an all-zero load."""
    load = [float(x) for x in load]
    mx = max(load)
    return (mx - sum(load) / len(load)) / mx if mx > 0 else 0.0


def worker_q_owned(blocks, owner, worker):
    """(seq, idx) rows of the blocks a worker owns, in block order."""
    return [(int(b[0]), int(b[1])) for b, o in zip(blocks, owner) if o == worker]


# --------------------------------------------------------------------------
# data flow -> bipartite multigraph
# --------------------------------------------------------------------------
def comm_edges(blocks, owner, causal=1):
    """Edges (src worker, dst worker, kv block), ordered by (kv block, dst).

    Query block (s, i) owned by w depends on KV blocks (s, j), j <= i under a causal mask,
    every j otherwise; if the KV block's owner u differs from w the block travels u -> w,
    once per (block, w).
    """
    by_seq = {}
    for b, blk in enumerate(blocks):
        by_seq.setdefault(int(blk[0]), []).append(b)
    edges = set()
    for qb, q in enumerate(blocks):
        w = owner[qb]
        for kb in by_seq[int(q[0])]:
            if causal and int(blocks[kb][1]) > int(q[1]):
                continue
            u = owner[kb]
            if u != w:
                edges.add((kb, w, u))
    out = sorted(edges)
    return [(u, w, kb) for kb, w, u in out]


def max_degree(src, dst, n_workers):
    """Delta of the bipartite multigraph: the largest send or receive count of any worker."""
    send, recv = [0] * n_workers, [0] * n_workers
    for u, w in zip(src, dst):
        send[u] += 1
        recv[w] += 1
    return max(send + recv) if len(src) else 0


# --------------------------------------------------------------------------
# congestion-free solver
# --------------------------------------------------------------------------
def solve_matchings(src, dst, n_workers):
    """Splits the edges into Delta matchings the way the appendix proof constructs them.

    Returns (stage [E], Delta).  1) pad to a Delta-regular multigraph by adding edges between a
    send node and a receive node that both have degree < Delta; 2) Delta times: take a perfect
    matching (library Hopcroft-Karp on the support graph), give it the next stage number and
    remove one copy of each of its edges; 3) forget the padding.
    """
    E, N = len(src), int(n_workers)
    D = max_degree(src, dst, N)
    if E == 0:
        return [], 0
    send, recv = [0] * N, [0] * N
    # multiplicity table with the ids of the real edges behind each (u, w)
    ids = {}
    mult = np.zeros((N, N), dtype=np.int64)
    for e, (u, w) in enumerate(zip(src, dst)):
        ids.setdefault((u, w), []).append(e)
        mult[u, w] += 1
        send[u] += 1
        recv[w] += 1
    u, w = 0, 0
    while True:
        while u < N and send[u] == D:
            u += 1
        while w < N and recv[w] == D:
            w += 1
        if u == N or w == N:
            break
        k = min(D - send[u], D - recv[w])
        mult[u, w] += k          # padding: copies beyond len(ids[(u, w)])
        send[u] += k
        recv[w] += k
    assert all(x == D for x in send) and all(x == D for x in recv)
    stage = [-1] * E
    for t in range(D):
        match = maximum_bipartite_matching(csr_matrix((mult > 0).astype(np.int8)), perm_type="column")
        assert (match >= 0).all(), "a regular bipartite graph has a perfect matching"
        for uu in range(N):
            ww = int(match[uu])
            mult[uu, ww] -= 1
            real = ids.get((uu, ww))
            if real:                      # real copies are handed out before padding copies
                stage[real.pop()] = t
    assert all(s >= 0 for s in stage)
    return stage, D


def check_matchings(src, dst, stage, n_workers):
    """What makes a split congestion-free and optimal: every edge has one stage in [0, Delta), and
    within a stage no worker sends twice or receives twice (Lemma 1); Lemma 2 makes Delta the
    minimum, so using exactly Delta stages is optimal.  Returns Delta; raises AssertionError."""
    D = max_degree(src, dst, n_workers)
    assert len(stage) == len(src) == len(dst)
    seen_s, seen_r = set(), set()
    for u, w, t in zip(src, dst, stage):
        assert 0 <= t < D, "stage out of range"
        assert (t, u) not in seen_s, "a worker sends twice in one sub-stage"
        assert (t, w) not in seen_r, "a worker receives twice in one sub-stage"
        seen_s.add((t, u))
        seen_r.add((t, w))
    return D


def coalesce_stages(stage, c):
    """Bottom-up coalescer: sub-stages [k c, (k+1) c) form stage k; c <= 0 puts everything in stage 0."""
    return [t // c if c > 0 else 0 for t in stage]
