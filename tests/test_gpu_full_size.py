"""GPU parity at the benchmark's full sizes.

`_run(..., timed=True)` issues exactly the launches bench.py times: FCP_FLAG_DIRECT_SINGLE (| FCP_FLAG_O_F32 |
FCP_FLAG_BWD_SPILL_DS for the training step), fcp_block_attn_fwd_out -> fcp_merge_partials -> fcp_block_attn_bwd
(= D pass, dK/dV kernel that leaves dS in the workspace, dQ from that dS).  `timed=False` is the staged path without
those flags: every query block through the partial buffers and the merge, then fcp_bwd_preprocess + the dK/dV kernel
and the recomputing dQ kernel called one by one.  `timed="recompute"` is fcp_block_attn_bwd without the spill flag
(dQ kernel that forms D itself, then dK/dV), which `bench.py --bwd recompute` times.  The training step runs all three.

The fp64 oracle cannot evaluate these workloads whole in test time, so it is asked for outputs it
can compute one by one from the plain definition:
  * O / LSE / dQ of sampled query rows (each against every visible key of its sequence);
  * whole short sequences (all of O, LSE, dQ, dK, dV);
  * dK / dV of the last rows of long sequences (only the rows at or after them contribute);
and the rest is covered by properties that hold at any size: sum_j dK_j = 0 per sequence and KV
head, sum_j dV_j = sum of dO over the rows and heads that attend, no unwritten (NaN) output.
Bars as in test_gpu_parity.py."""
import sys
import time

import numpy as np
import pytest
import torch

from oracle import fcp_oracle as orc
from paper_2605_08524_amd import workloads
from paper_2605_08524_amd.harness import DevicePath

pytestmark = pytest.mark.gpu

TOL_ABS, TOL_REL, TOL_LSE = 2e-2, 1e-2, 1e-3
F32 = 1


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


class _Acc:
    """Accumulates max-abs and relative-L2 error over many pieces of one output."""

    def __init__(self, name):
        self.name, self.max_abs, self.num, self.den, self.n = name, 0.0, 0.0, 0.0, 0

    def add(self, got, ref):
        got = np.asarray(got, dtype=np.float64)
        assert got.shape == ref.shape, (self.name, got.shape, ref.shape)
        assert np.all(np.isfinite(got)), f"{self.name}: non-finite values"
        if ref.size:
            self.max_abs = max(self.max_abs, float(np.max(np.abs(got - ref))))
            self.num += float(np.sum((got - ref) ** 2))
            self.den += float(np.sum(ref * ref))
            self.n += ref.size

    def check(self, tol_abs=TOL_ABS, tol_rel=TOL_REL):
        rel = (self.num / self.den) ** 0.5 if self.den > 0 else 0.0
        _say(f"  {self.name}: {self.n} values, max-abs {self.max_abs:.3e}, rel-L2 {rel:.3e}")
        assert self.n > 0, self.name
        assert self.max_abs <= tol_abs, (self.name, self.max_abs)
        if tol_rel is not None:
            assert rel <= tol_rel, (self.name, rel)


def _seq_geometry(wl):
    """Per sequence: KV offset, and Q-buffer row of every owned position (-1 = not owned)."""
    bs = wl.block_size
    koff = np.concatenate([[0], np.cumsum(wl.seq_lens.astype(np.int64))])
    qrow = [None] * len(wl.seq_lens)
    owned = wl.q_owned
    if owned is None:
        for s, L in enumerate(wl.seq_lens):
            qrow[s] = koff[s] + np.arange(int(L))
        return koff, qrow
    cur = 0
    for s, L in enumerate(wl.seq_lens):
        qrow[s] = np.full(int(L), -1, dtype=np.int64)
    for s, i in owned:
        L = int(wl.seq_lens[s])
        lo = int(i) * bs
        n = min(bs, L - lo)
        qrow[int(s)][lo:lo + n] = cur + np.arange(n)
        cur += n
    return koff, qrow


def _rows_check(wl, host, seq, positions, accs, backward, koff, qrow):
    """Oracle for sampled query positions of one sequence, one KV head at a time (K and V of a
    head are converted to fp64 once).  Checks O, LSE and (backward) dQ of those rows."""
    L = int(wl.seq_lens[seq])
    G = wl.n_q_heads // wl.n_kv_heads
    positions = np.asarray(sorted(set(int(p) for p in positions)))
    rows = qrow[seq][positions]
    assert np.all(rows >= 0)
    hi = int(positions.max()) + 1 if wl.causal else L
    k0 = int(koff[seq])
    q, k, v = wl.q(), wl.k(), wl.v()
    for g in range(wl.n_kv_heads):
        kh = orc.bf16_to_f64(k[k0:k0 + hi, g:g + 1])
        vh = orc.bf16_to_f64(v[k0:k0 + hi, g:g + 1])
        qh = orc.bf16_to_f64(q[rows][:, g * G:(g + 1) * G])
        o, lse = orc.attention_fwd_seq(qh, kh, vh, bool(wl.causal), None, q_pos=positions, k_pos=np.arange(hi))
        accs["o"].add(host["o"][rows][:, g * G:(g + 1) * G], o)
        accs["lse"].add(host["lse"][rows][:, g * G:(g + 1) * G], lse)
        if backward:
            doh = orc.bf16_to_f64(wl.d_o()[rows][:, g * G:(g + 1) * G])
            dq, _, _ = orc.attention_bwd_seq(qh, kh, vh, doh, bool(wl.causal), None, q_pos=positions, k_pos=np.arange(hi))
            accs["dq"].add(host["dq"][rows][:, g * G:(g + 1) * G], dq)


def _whole_seq_check(wl, host, seq, accs, backward, koff, qrow):
    L = int(wl.seq_lens[seq])
    k0 = int(koff[seq])
    rows = qrow[seq]
    assert np.all(rows >= 0)
    qs = orc.bf16_to_f64(wl.q()[rows])
    ks = orc.bf16_to_f64(wl.k()[k0:k0 + L])
    vs = orc.bf16_to_f64(wl.v()[k0:k0 + L])
    o, lse = orc.attention_fwd_seq(qs, ks, vs, bool(wl.causal))
    accs["o"].add(host["o"][rows], o)
    accs["lse"].add(host["lse"][rows], lse)
    if backward:
        dq, dk, dv = orc.attention_bwd_seq(qs, ks, vs, orc.bf16_to_f64(wl.d_o()[rows]), bool(wl.causal))
        accs["dq"].add(host["dq"][rows], dq)
        accs["dk"].add(host["dk"][k0:k0 + L], dk)
        accs["dv"].add(host["dv"][k0:k0 + L], dv)


def _tail_check(wl, host, seq, n_tail, accs, koff, qrow):
    """Last n_tail rows of a causal sequence: only they contribute to dK/dV of the last n_tail keys."""
    L = int(wl.seq_lens[seq])
    k0 = int(koff[seq])
    start = L - n_tail
    pos = np.arange(start, L)
    rows = qrow[seq][pos]
    assert np.all(rows >= 0)
    G = wl.n_q_heads // wl.n_kv_heads
    for g in range(wl.n_kv_heads):
        kh = orc.bf16_to_f64(wl.k()[k0:k0 + L, g:g + 1])
        vh = orc.bf16_to_f64(wl.v()[k0:k0 + L, g:g + 1])
        qh = orc.bf16_to_f64(wl.q()[rows][:, g * G:(g + 1) * G])
        doh = orc.bf16_to_f64(wl.d_o()[rows][:, g * G:(g + 1) * G])
        dq, dk, dv = orc.attention_bwd_seq(qh, kh, vh, doh, True, None, q_pos=pos, k_pos=np.arange(L))
        accs["dq"].add(host["dq"][rows][:, g * G:(g + 1) * G], dq)
        accs["dk"].add(host["dk"][k0 + start:k0 + L, g:g + 1], dk[start:])
        accs["dv"].add(host["dv"][k0 + start:k0 + L, g:g + 1], dv[start:])


DIRECT = 2   # FCP_FLAG_DIRECT_SINGLE
SPILL = 16   # FCP_FLAG_BWD_SPILL_DS


def _run(wl, backward, flags, timed=True, packed=False):
    dev = torch.device("cuda:0")
    t0 = time.time()
    if timed:
        flags |= DIRECT
    if timed is True and backward:
        flags |= SPILL
    dp = DevicePath(wl, dev, flags=flags, backward=backward, packed=packed)
    _say(f"  inputs generated and uploaded in {time.time() - t0:.1f} s; "
         f"{len(dp.plan['pairs'])} pairs, {len(dp.plan['slots'])} slots, {dp.problem.n_slot_rows} partial rows")
    dp.fwd()
    dp.merge()
    if backward and timed:
        dp.bwd()
    elif backward:
        dp.bwd_pre()
        dp.bwd_dkdv()
        dp.bwd_dq()
    torch.cuda.synchronize(dev)
    p = dp.problem
    host = dict(o=dp.o[: p.t_q].float().cpu().numpy(), lse=dp.lse[: p.t_q].cpu().numpy())
    if backward:
        host.update(dq=dp.dq[: p.t_q].cpu().numpy(), dk=dp.dk[: p.t_kv].cpu().numpy(), dv=dp.dv[: p.t_kv].cpu().numpy())
    # partial buffers: every row written (no NaN left from the poison fill); with FCP_FLAG_DIRECT_SINGLE the rows
    # of a query block's only slot are left alone on purpose (its result went straight to the final outputs)
    multi = np.ones(len(dp.plan["slots"]), dtype=bool)
    if timed and len(multi):
        cnt = np.bincount(dp.plan["slots"][:, 0], minlength=len(dp.plan["q_blocks"]))
        multi = cnt[dp.plan["slots"][:, 0]] > 1
    rows = np.zeros(max(1, p.n_slot_rows), dtype=bool)
    for sl in dp.plan["slots"][multi]:
        rows[sl[3]:sl[3] + dp.plan["q_blocks"][sl[0], 3]] = True
    sel = torch.from_numpy(rows).to(dev)
    assert bool(torch.isfinite(dp.o_part[sel]).all()), "unwritten partial rows"
    lp = dp.lse_part[sel]
    assert bool((torch.isfinite(lp) | (lp == float("-inf"))).all())
    plan = dp.plan
    del dp
    torch.cuda.empty_cache()
    return host, plan


def _tables_exact(wl, plan):
    ref = orc.plan_blocks(wl.seq_lens, wl.block_size, wl.causal, wl.coalesce, wl.q_owned)
    for key in ("kv_blocks", "q_blocks", "pairs", "slots"):
        assert np.array_equal(ref[key], plan[key]), key
    assert ref["n_slot_rows"] == plan["n_slot_rows"]


def _gradient_sum_properties(wl, host, koff):
    """Hold for any mask and size: the rows of dS sum to zero, so sum_j dK_j = 0 per sequence and KV head;
    the rows of P sum to one, so sum_j dV_j = sum of dO over the sequence's rows and the heads of the group."""
    G = wl.n_q_heads // wl.n_kv_heads
    for s, L in enumerate(wl.seq_lens):
        k0, L = int(koff[s]), int(L)
        if L == 0:
            continue
        dk, dv = host["dk"][k0:k0 + L].astype(np.float64), host["dv"][k0:k0 + L].astype(np.float64)
        assert np.max(np.abs(dk.sum(axis=0))) <= 2e-3 * np.abs(dk).sum(axis=0).max() + 1e-3, f"sum dK != 0 in seq {s}"
        do = workloads.bf16_to_f32(wl.d_o()[k0:k0 + L]).astype(np.float64)
        want = do.reshape(L, wl.n_kv_heads, G, wl.head_dim).sum(axis=(0, 2))
        assert np.max(np.abs(dv.sum(axis=0) - want)) <= 2e-3 * np.abs(dv).sum(axis=0).max() + 1e-3, f"sum dV in seq {s}"


@pytest.mark.timeout(900)
@pytest.mark.parametrize("seed,timed", [(0, True), (1, True), (2, True), (0, "recompute"), (0, False)])
def test_config5_training_step_full_size(seed, timed):
    wl = workloads.make_workload(5, seed)
    _say(f"case {wl.name} seed={seed} {'launches as timed: ' + str(timed) if timed else 'staged launches'}: {len(wl.seq_lens)} sequences, "
         f"lengths {sorted(int(x) for x in wl.seq_lens)}")
    host, plan = _run(wl, True, F32, timed)
    _training_step_checks(wl, host, plan)


def _training_step_checks(wl, host, plan, whole_up_to=1300, n_rows=24):
    _tables_exact(wl, plan)
    for name in ("o", "lse", "dq", "dk", "dv"):
        assert np.all(np.isfinite(host[name])), f"{name}: unwritten or non-finite rows"
    koff, qrow = _seq_geometry(wl)
    accs = {n: _Acc(n) for n in ("o", "lse", "dq", "dk", "dv")}
    rng = np.random.default_rng(123)
    t0 = time.time()
    for s, L in enumerate(wl.seq_lens):
        L = int(L)
        if L <= whole_up_to:
            _whole_seq_check(wl, host, s, accs, True, koff, qrow)
        else:
            _tail_check(wl, host, s, 96, accs, koff, qrow)
            _rows_check(wl, host, s, rng.integers(0, L - 96, size=n_rows), accs, True, koff, qrow)
        _say(f"  seq {s} (L={L}) checked, {time.time() - t0:.0f} s")
    accs["o"].check()
    accs["lse"].check(TOL_LSE, None)
    accs["dq"].check()
    accs["dk"].check()
    accs["dv"].check()
    _gradient_sum_properties(wl, host, koff)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("block,coalesce", [(4096, 1), (4096, 16), (8192, 1), (8192, 16)])
def test_training_step_with_large_blocks(block, coalesce):
    """The block sizes at the upper end of the block-size sweep (the paper's system runs 4K-token blocks): the
    training batch cut into 4096- and 8192-token blocks, one partial per KV block (c = 1: the merge runs) and
    coalesce degree 16, forward and backward in the timed launch configuration."""
    wl = workloads.make_workload(5, 0)
    wl.block_size, wl.coalesce = block, coalesce
    wl.name += f"-block{block}-c{coalesce}"
    _say(f"case {wl.name}: {len(wl.seq_lens)} sequences")
    host, plan = _run(wl, True, F32, True)
    assert plan["q_blocks"][:, 3].max() > 2048
    _training_step_checks(wl, host, plan, whole_up_to=700, n_rows=10)


@pytest.mark.timeout(600)
def test_config2_forward_full_size_bf16_output():
    wl = workloads.make_workload(2, 1)
    _say(f"case {wl.name} seed=1: {len(wl.seq_lens)} sequences")
    host, plan = _run(wl, False, 0)
    _tables_exact(wl, plan)
    koff, qrow = _seq_geometry(wl)
    accs = {n: _Acc(n) for n in ("o", "lse")}
    rng = np.random.default_rng(7)
    for s, L in enumerate(wl.seq_lens):
        L = int(L)
        if L <= 1100:
            _whole_seq_check(wl, host, s, accs, False, koff, qrow)
        else:
            pos = np.concatenate([rng.integers(0, L, size=24), [0, L - 1, 1023, 1024]])
            _rows_check(wl, host, s, pos[pos < L], accs, False, koff, qrow)
    accs["o"].check()
    accs["lse"].check(TOL_LSE, None)


_WL3 = []


def _config3():
    """The long-sequence share, generated once for the tests that use it (a minute of host time)."""
    if not _WL3:
        _WL3.append(workloads.make_workload(3, 0))
    return _WL3[0]


@pytest.mark.timeout(1200)
def test_config3_long_sequence_share_running_merge():
    """The long-sequence share without any partial buffer: about 32 stages (16 KV blocks each), every stage one launch
    that folds its slots into the running (O, LSE) in place; sampled rows against the oracle."""
    from paper_2605_08524_amd.harness import run_running_forward
    wl = _config3()
    _say(f"case {wl.name} with a running result: 1M-token sequence, {len(wl.q_owned)} owned query blocks")
    t0 = time.time()
    res = run_running_forward(wl, torch.device("cuda:0"))
    _say(f"  {res['n_stages']} stages in {time.time() - t0:.1f} s (inputs included)")
    assert res["n_stages"] == -(-(int(wl.q_owned[:, 1].max()) + 1) // wl.coalesce) >= 30
    _tables_exact(wl, res["plan"])
    assert np.all(np.isfinite(res["o"])) and np.all(np.isfinite(res["lse"]))
    koff, qrow = _seq_geometry(wl)
    accs = {n: _Acc(n) for n in ("o", "lse")}
    rng = np.random.default_rng(17)
    bs = wl.block_size
    blocks = wl.q_owned[rng.choice(len(wl.q_owned), size=12, replace=False), 1]
    pos = [int(b) * bs + int(rng.integers(0, bs)) for b in blocks]
    last = int(wl.q_owned[-1, 1]) * bs
    pos += [last, last + bs - 1]                        # first and last row of the last owned block (it goes through every stage)
    _rows_check(wl, res, 0, pos, accs, False, koff, qrow)
    accs["o"].check()
    accs["lse"].check(TOL_LSE, None)


@pytest.mark.timeout(1200)
def test_config3_long_sequence_share_sampled():
    wl = _config3()
    _say(f"case {wl.name}: 1M-token sequence, {len(wl.q_owned)} owned query blocks")
    host, plan = _run(wl, False, 0)
    _tables_exact(wl, plan)
    assert len(plan["pairs"]) == 32 * 513
    assert np.all(np.isfinite(host["o"])) and np.all(np.isfinite(host["lse"]))
    koff, qrow = _seq_geometry(wl)
    accs = {n: _Acc(n) for n in ("o", "lse")}
    rng = np.random.default_rng(11)
    bs = wl.block_size
    blocks = wl.q_owned[rng.choice(len(wl.q_owned), size=20, replace=False), 1]
    pos = [int(b) * bs + int(rng.integers(0, bs)) for b in blocks]
    first = int(wl.q_owned[0, 1]) * bs
    pos += [first, first + bs - 1]                      # first and last row of the first owned block
    t0 = time.time()
    _rows_check(wl, host, 0, pos, accs, False, koff, qrow)
    _say(f"  oracle rows in {time.time() - t0:.0f} s")
    accs["o"].check()
    accs["lse"].check(TOL_LSE, None)


@pytest.mark.timeout(900)
def test_config4_multimodal_mix_sampled():
    wl = workloads.make_workload(4, 0)
    _say(f"case {wl.name}: {len(wl.seq_lens)} sequences, long one {int(wl.seq_lens[-1])} tokens")
    host, plan = _run(wl, False, 0)
    _tables_exact(wl, plan)
    assert np.all(np.isfinite(host["o"])) and np.all(np.isfinite(host["lse"]))
    koff, qrow = _seq_geometry(wl)
    accs = {n: _Acc(n) for n in ("o", "lse")}
    rng = np.random.default_rng(5)
    for s in rng.choice(len(wl.seq_lens) - 1, size=12, replace=False):
        _whole_seq_check(wl, host, int(s), accs, False, koff, qrow)
    long_seq = len(wl.seq_lens) - 1
    owned_pos = np.nonzero(qrow[long_seq] >= 0)[0]
    pos = list(rng.choice(owned_pos, size=16, replace=False)) + [int(owned_pos[0]), int(owned_pos[-1])]
    _rows_check(wl, host, long_seq, pos, accs, False, koff, qrow)
    accs["o"].check()
    accs["lse"].check(TOL_LSE, None)


@pytest.mark.timeout(900)
def test_config4_multimodal_mix_packed_blocks():
    """Config 4 planned with fcp_plan_blocks_packed (block costs -> scheduling units -> packed plan, all in the library):
    tables against the oracle's chain, then forward and backward on the timed launches; every member of a packed block
    is checked whole (O, LSE, dQ, dK, dV), with some unpacked short sequences and sampled rows of the long one."""
    from oracle import fcp_sched_oracle as sch
    wl = workloads.make_workload(4, 0)
    _say(f"case {wl.name} packed: {len(wl.seq_lens)} sequences, long one {int(wl.seq_lens[-1])} tokens")
    got, plan = _run(wl, True, F32, packed=True)
    flat = orc.plan_blocks(wl.seq_lens, wl.block_size, wl.causal, 0)["kv_blocks"]
    unit, _, _ = sch.pack_units(flat, [int(b[3]) for b in flat], [0] * len(flat), wl.block_size)
    ref = orc.plan_blocks_packed(wl.seq_lens, wl.block_size, wl.causal, wl.coalesce, wl.q_owned, unit)
    for key in ("kv_blocks", "q_blocks", "pairs", "slots", "segments"):
        assert np.array_equal(ref[key], plan[key]), key
    members = sorted(set(int(s) for _, s, _, _ in ref["segments"]))
    assert len(members) >= 20
    # back to the sequence-major layout that the sampling helpers index
    kv_src, q_src = orc.packed_row_maps(ref, wl.seq_lens, wl.block_size, wl.q_owned)
    host = {}
    for name, src in (("o", q_src), ("lse", q_src), ("dq", q_src), ("dk", kv_src), ("dv", kv_src)):
        assert np.all(np.isfinite(got[name]) | (np.isneginf(got[name]) if name == "lse" else False)), name
        host[name] = np.empty_like(got[name])
        host[name][src] = got[name]
    koff, qrow = _seq_geometry(wl)
    accs = {n: _Acc(n) for n in ("o", "lse", "dq", "dk", "dv")}
    rng = np.random.default_rng(6)
    others = [int(s) for s in rng.permutation(len(wl.seq_lens) - 1) if int(s) not in members][:6]
    for s in members + others:
        _whole_seq_check(wl, host, s, accs, True, koff, qrow)
    long_seq = len(wl.seq_lens) - 1
    owned_pos = np.nonzero(qrow[long_seq] >= 0)[0]
    pos = list(rng.choice(owned_pos, size=8, replace=False)) + [int(owned_pos[0]), int(owned_pos[-1])]
    _rows_check(wl, host, long_seq, pos, accs, True, koff, qrow)
    for n in ("o", "dq", "dk", "dv"):
        accs[n].check()
    accs["lse"].check(TOL_LSE, None)


@pytest.mark.timeout(900)
def test_noncausal_batch_with_64_query_heads_full_size():
    """The packed 64K-token batch without a causal mask (every pair FULL, ragged last KV block of each
    sequence) at 64 query / 8 KV heads, the head shape of the paper's model: forward and backward."""
    base = workloads.make_workload(2, 2)
    wl = workloads.custom_workload(base.seq_lens, 1024, causal=0, coalesce=16, n_q_heads=64, n_kv_heads=8,
                                   head_dim=128, seed=2, name="noncausal-64q8kv")
    _say(f"case {wl.name}: {len(wl.seq_lens)} sequences, lengths {sorted(int(x) for x in wl.seq_lens)}")
    host, plan = _run(wl, True, F32)
    _tables_exact(wl, plan)
    assert (plan["pairs"][:, 2] == 0).all()
    for name in ("o", "lse", "dq", "dk", "dv"):
        assert np.all(np.isfinite(host[name])), f"{name}: unwritten or non-finite rows"
    koff, qrow = _seq_geometry(wl)
    accs = {n: _Acc(n) for n in ("o", "lse", "dq", "dk", "dv")}
    rng = np.random.default_rng(321)
    t0 = time.time()
    for s, L in enumerate(wl.seq_lens):
        L = int(L)
        if L <= 1000:
            _whole_seq_check(wl, host, s, accs, True, koff, qrow)
        else:
            _rows_check(wl, host, s, np.concatenate([rng.integers(0, L, size=10), [0, L - 1]]), accs, True, koff, qrow)
        _say(f"  seq {s} (L={L}) checked, {time.time() - t0:.0f} s")
    accs["o"].check()
    accs["lse"].check(TOL_LSE, None)
    accs["dq"].check()
    if accs["dk"].n:
        accs["dk"].check()
        accs["dv"].check()
    _gradient_sum_properties(wl, host, koff)
