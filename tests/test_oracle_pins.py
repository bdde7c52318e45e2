"""Pins for the CPU oracle: each check ties it to something other than itself
(brute force, closed forms, a library routine, finite differences, invariants,
the numbers printed in the paper's Zig-Zag figure caption)."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import fcp_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(rng, *shape):
    return rng.standard_normal(shape)


def _brute_fwd(q, k, v, causal, scale):
    """Triple-loop softmax attention in Python floats."""
    Lq, Hq, d = q.shape
    Lk, Hkv, _ = k.shape
    o = [[[0.0] * d for _ in range(Hq)] for _ in range(Lq)]
    lse = [[0.0] * Hq for _ in range(Lq)]
    for i in range(Lq):
        for h in range(Hq):
            g = h // (Hq // Hkv)
            js = [j for j in range(Lk) if (not causal or j <= i)]
            s = [scale * sum(float(q[i, h, c]) * float(k[j, g, c]) for c in range(d)) for j in js]
            tot = sum(math.exp(x) for x in s)
            lse[i][h] = math.log(tot)
            for c in range(d):
                o[i][h][c] = sum(math.exp(x) / tot * float(v[j, g, c]) for x, j in zip(s, js))
    return np.array(o), np.array(lse)


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("hq,hkv", [(2, 2), (4, 2), (4, 1)])
def test_fwd_matches_brute_force(causal, hq, hkv):
    rng = np.random.default_rng(7)
    L, d = 11, 5
    q, k, v = _rand(rng, L, hq, d), _rand(rng, L, hkv, d), _rand(rng, L, hkv, d)
    o, lse = orc.attention_fwd_seq(q, k, v, causal, row_chunk=4)
    ob, lb = _brute_fwd(q, k, v, causal, 1 / math.sqrt(d))
    assert np.max(np.abs(o - ob)) < 1e-12
    assert np.max(np.abs(lse - lb)) < 1e-12


def test_fwd_rows_of_p_sum_to_one():
    rng = np.random.default_rng(1)
    L, H, d = 37, 3, 8
    q, k = _rand(rng, L, H, d), _rand(rng, L, H, d)
    o, _ = orc.attention_fwd_seq(q, k, np.ones((L, H, d)), True)
    assert np.max(np.abs(o - 1.0)) < 1e-14


def test_fwd_closed_form_equal_keys():
    rng = np.random.default_rng(2)
    L, H, d = 23, 2, 6
    q, v = _rand(rng, L, H, d), _rand(rng, L, H, d)
    k0 = _rand(rng, H, d)
    k = np.broadcast_to(k0, (L, H, d)).copy()
    o, lse = orc.attention_fwd_seq(q, k, v, True)
    scale = 1 / math.sqrt(d)
    for i in range(L):
        assert np.allclose(o[i], v[: i + 1].mean(axis=0), atol=1e-13)
        assert np.allclose(lse[i], scale * np.sum(q[i] * k0, axis=-1) + math.log(i + 1), atol=1e-13)


def test_fwd_single_token():
    rng = np.random.default_rng(3)
    q, k, v = _rand(rng, 1, 4, 8), _rand(rng, 1, 2, 8), _rand(rng, 1, 2, 8)
    o, lse = orc.attention_fwd_seq(q, k, v, True)
    assert np.allclose(o[0], np.repeat(v[0], 2, axis=0), atol=0)
    assert np.allclose(lse[0], np.sum(q[0] * np.repeat(k[0], 2, axis=0), -1) / math.sqrt(8), atol=1e-15)


def _sdpa(q, k, v, causal):
    Hq, Hkv = q.shape[1], k.shape[1]
    tq = torch.tensor(q).permute(1, 0, 2)[None]
    tk = torch.tensor(k).permute(1, 0, 2)[None].repeat_interleave(Hq // Hkv, dim=1)
    tv = torch.tensor(v).permute(1, 0, 2)[None].repeat_interleave(Hq // Hkv, dim=1)
    return tq, tk, tv


@pytest.mark.parametrize("causal", [True, False])
def test_fwd_matches_library_sdpa(causal):
    rng = np.random.default_rng(4)
    L, Hq, Hkv, d = 70, 4, 2, 16
    q, k, v = _rand(rng, L, Hq, d), _rand(rng, L, Hkv, d), _rand(rng, L, Hkv, d)
    tq, tk, tv = _sdpa(q, k, v, causal)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=causal)[0].permute(1, 0, 2).numpy()
    o, _ = orc.attention_fwd_seq(q, k, v, causal, row_chunk=32)
    assert np.max(np.abs(o - ref)) < 1e-12


@pytest.mark.parametrize("causal", [True, False])
def test_bwd_matches_library_autograd(causal):
    rng = np.random.default_rng(5)
    L, Hq, Hkv, d = 45, 4, 2, 8
    q, k, v, do = _rand(rng, L, Hq, d), _rand(rng, L, Hkv, d), _rand(rng, L, Hkv, d), _rand(rng, L, Hq, d)
    tq = torch.tensor(q, requires_grad=True)
    tk = torch.tensor(k, requires_grad=True)
    tv = torch.tensor(v, requires_grad=True)
    a = tq.permute(1, 0, 2)[None]
    b = tk.permute(1, 0, 2)[None].repeat_interleave(Hq // Hkv, dim=1)
    c = tv.permute(1, 0, 2)[None].repeat_interleave(Hq // Hkv, dim=1)
    out = torch.nn.functional.scaled_dot_product_attention(a, b, c, is_causal=causal)[0].permute(1, 0, 2)
    (out * torch.tensor(do)).sum().backward()
    dq, dk, dv = orc.attention_bwd_seq(q, k, v, do, causal, row_chunk=16)
    assert np.max(np.abs(dq - tq.grad.numpy())) < 1e-12
    assert np.max(np.abs(dk - tk.grad.numpy())) < 1e-12
    assert np.max(np.abs(dv - tv.grad.numpy())) < 1e-12


def test_bwd_finite_differences():
    rng = np.random.default_rng(6)
    L, Hq, Hkv, d = 9, 2, 1, 4
    q, k, v, do = _rand(rng, L, Hq, d), _rand(rng, L, Hkv, d), _rand(rng, L, Hkv, d), _rand(rng, L, Hq, d)
    dq, dk, dv = orc.attention_bwd_seq(q, k, v, do, True)

    def loss(q_, k_, v_):
        return float(np.sum(orc.attention_fwd_seq(q_, k_, v_, True)[0] * do))

    eps = 1e-6
    for arr, grad, which in ((q, dq, 0), (k, dk, 1), (v, dv, 2)):
        num = np.zeros_like(arr)
        for idx in np.ndindex(arr.shape):
            hi, lo = arr.copy(), arr.copy()
            hi[idx] += eps
            lo[idx] -= eps
            args_hi = [q, k, v]
            args_lo = [q, k, v]
            args_hi[which], args_lo[which] = hi, lo
            num[idx] = (loss(*args_hi) - loss(*args_lo)) / (2 * eps)
        assert np.max(np.abs(num - grad)) / max(1.0, np.max(np.abs(grad))) < 1e-6


def test_bwd_invariants():
    rng = np.random.default_rng(8)
    L, Hq, Hkv, d = 33, 4, 2, 8
    q, k, v, do = _rand(rng, L, Hq, d), _rand(rng, L, Hkv, d), _rand(rng, L, Hkv, d), _rand(rng, L, Hq, d)
    dq, dk, dv = orc.attention_bwd_seq(q, k, v, do, True)
    # softmax is shift invariant along the key axis: the key gradients of a KV head sum to zero
    assert np.max(np.abs(dk.sum(axis=0))) < 1e-12
    # rows of P sum to one: dV summed over keys equals dO summed over rows and the group's heads
    want = do.reshape(L, Hkv, Hq // Hkv, d).sum(axis=(0, 2))
    assert np.max(np.abs(dv.sum(axis=0) - want)) < 1e-12
    z = orc.attention_bwd_seq(q, k, v, np.zeros_like(do), True)
    assert all(np.all(t == 0) for t in z)


def _bits(rng, *shape):
    from paper_2605_08524_amd.workloads import bf16_bits
    return bf16_bits(rng.standard_normal(shape).astype(np.float32))


@pytest.mark.parametrize("bs,c", [(4, 1), (5, 2), (8, 0), (3, 3), (64, 16)])
@pytest.mark.parametrize("causal", [1, 0])
def test_block_partials_merge_to_whole(bs, c, causal):
    """Associativity stated in section "Context Parallelism": partial results over
    slices of the context reduce to the whole-sequence result."""
    rng = np.random.default_rng(9)
    seq_lens = [13, 1, 8, 0, 21, 5]
    T, Hq, Hkv, d = sum(seq_lens), 4, 2, 8
    q, k, v = _bits(rng, T, Hq, d), _bits(rng, T, Hkv, d), _bits(rng, T, Hkv, d)
    plan = orc.plan_blocks(seq_lens, bs, causal, c)
    op, lp = orc.partial_fwd(q, k, v, plan, bs, causal)
    o, lse = orc.merge_partials(op, lp, plan)
    ow, lw = orc.worker_fwd(q, k, v, seq_lens, bs, causal)
    assert np.max(np.abs(o - ow)) < 1e-12
    assert np.max(np.abs(lse - lw)) < 1e-12


def test_share_of_owned_blocks():
    rng = np.random.default_rng(10)
    seq_lens, bs = [19, 7, 30], 4
    T, Hq, Hkv, d = sum(seq_lens), 2, 1, 4
    k, v = _bits(rng, T, Hkv, d), _bits(rng, T, Hkv, d)
    qfull, dofull = _bits(rng, T, Hq, d), _bits(rng, T, Hq, d)
    full = orc.plan_blocks(seq_lens, bs, 1, 2)
    owned_a = [(0, 1), (0, 4), (2, 0), (2, 7)]
    owned_b = [(int(s), int(i)) for s, i, _, _ in full["kv_blocks"] if (int(s), int(i)) not in owned_a]

    def rows_of(owned):
        r = []
        for s, i in owned:
            base = sum(seq_lens[:s]) + i * bs
            r += list(range(base, min(base + bs, sum(seq_lens[: s + 1]))))
        return np.array(r)

    ofull, lfull = orc.worker_fwd(qfull, k, v, seq_lens, bs, 1)
    dqf, dkf, dvf = orc.worker_bwd(qfull, k, v, dofull, seq_lens, bs, 1)
    dk_sum = np.zeros_like(dkf)
    dv_sum = np.zeros_like(dvf)
    for owned in (owned_a, owned_b):
        rows = rows_of(owned)
        plan = orc.plan_blocks(seq_lens, bs, 1, 2, owned)
        assert plan["q_blocks"][:, 3].sum() == len(rows)
        o, lse = orc.worker_fwd(qfull[rows], k, v, seq_lens, bs, 1, owned)
        assert np.max(np.abs(o - ofull[rows])) < 1e-13 and np.max(np.abs(lse - lfull[rows])) < 1e-13
        op, lp = orc.partial_fwd(qfull[rows], k, v, plan, bs, 1)
        om, lm = orc.merge_partials(op, lp, plan)
        assert np.max(np.abs(om - ofull[rows])) < 1e-12 and np.max(np.abs(lm - lfull[rows])) < 1e-12
        sample = np.arange(0, len(rows), 3)
        orow, lrow = orc.rows_fwd(qfull[rows], k, v, seq_lens, bs, plan, sample, 1)
        assert np.max(np.abs(orow - ofull[rows][sample])) < 1e-13
        assert np.max(np.abs(lrow - lfull[rows][sample])) < 1e-13
        dq, dk, dv = orc.worker_bwd(qfull[rows], k, v, dofull[rows], seq_lens, bs, 1, owned)
        assert np.max(np.abs(dq - dqf[rows])) < 1e-12
        dk_sum += dk
        dv_sum += dv
    assert np.max(np.abs(dk_sum - dkf)) < 1e-12 and np.max(np.abs(dv_sum - dvf)) < 1e-12


def test_merge_handles_empty_partials():
    plan = orc.plan_blocks([4], 2, 1, 1)
    n = plan["n_slot_rows"]
    o = np.ones((n, 1, 2))
    lse = np.full((n, 1), -np.inf)
    om, lm = orc.merge_partials(o, lse, plan)
    assert np.all(om == 0) and np.all(np.isneginf(lm))
    # q block 1 has two slots; make the first one empty, the second one carries the result
    lse2 = np.zeros((n, 1))
    r_first = int(plan["slots"][1][3])
    lse2[r_first:r_first + 2] = -np.inf
    o2 = np.arange(n * 2, dtype=np.float64).reshape(n, 1, 2)
    om, lm = orc.merge_partials(o2, lse2, plan)
    r_second = int(plan["slots"][2][3])
    assert np.array_equal(om[2:4], o2[r_second:r_second + 2]) and np.all(lm[2:4] == 0)


def _golden():
    out = {}
    with open(os.path.join(GOLDEN, "zigzag_figure_counts.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k_, v_ = line.split()
                out[k_] = int(v_)
    return out


def test_planner_zigzag_figure_counts():
    g = _golden()
    n, bs = g["n_blocks"], 16
    plan = orc.plan_blocks([n * bs], bs, 1, 1)
    pairs = plan["pairs"]
    qi = g["q_index"]
    mine = pairs[pairs[:, 0] == qi]
    assert len(mine) == g["kv_blocks_needed_by_q"]
    assert (mine[:, 2] == orc.DIAG).sum() == 1 and (mine[:, 2] == orc.FULL).sum() == len(mine) - 1
    later = pairs[(pairs[:, 1] == qi) & (pairs[:, 0] != qi)]
    assert len(later) == g["later_q_blocks_needing_kv"]
    assert len(pairs) == n * (n + 1) // 2 and (pairs[:, 2] == orc.DIAG).sum() == n
    # zig-zag partners (i, n-1-i) carry equal work: pairs(i) + pairs(n-1-i) = n + 1
    for i in range(n // 2):
        assert (pairs[:, 0] == i).sum() + (pairs[:, 0] == n - 1 - i).sum() == n + 1


def test_planner_quadratic_compute_ratio():
    g = _golden()
    nnz = []
    for L in (g["long_len"], g["short_len"]):
        plan = orc.plan_blocks([L], 1024, 1, 16)
        assert orc.pair_nnz(plan) == L * (L + 1) // 2
        nnz.append(orc.pair_nnz(plan))
    assert abs(nnz[0] / nnz[1] - g["compute_ratio"]) / g["compute_ratio"] < 1e-3


@pytest.mark.parametrize("causal", [1, 0])
@pytest.mark.parametrize("c", [0, 1, 2, 16])
def test_planner_brute_force_coverage(causal, c):
    """Every visible (query token, key token) entry is covered by exactly one pair,
    masked entries by none; table bookkeeping is consistent."""
    seq_lens, bs = [10, 3, 0, 17, 4, 1], 4
    owned = None
    plan = orc.plan_blocks(seq_lens, bs, causal, c, owned)
    kvb, qb, pairs, slots = plan["kv_blocks"], plan["q_blocks"], plan["pairs"], plan["slots"]
    assert kvb[:, 3].sum() == sum(seq_lens) and np.array_equal(kvb, qb)
    assert np.array_equal(kvb[:, 2], np.concatenate([[0], np.cumsum(kvb[:-1, 3])]))
    T = sum(seq_lens)
    seq_of = np.repeat(np.arange(len(seq_lens)), seq_lens)
    pos_of = np.concatenate([np.arange(L) for L in seq_lens])
    want = (seq_of[:, None] == seq_of[None, :])
    if causal:
        want &= pos_of[None, :] <= pos_of[:, None]
    got = np.zeros((T, T), dtype=np.int64)
    for q_, k_, kind, slot in pairs:
        _, _, qs, ql = qb[q_]
        _, _, ks, kl = kvb[k_]
        blk = np.ones((ql, kl), dtype=np.int64)
        if kind == orc.DIAG:
            assert q_ == k_ or (qb[q_][0] == kvb[k_][0] and qb[q_][1] == kvb[k_][1])
            blk = np.tril(blk)
        got[qs:qs + ql, ks:ks + kl] += blk
        assert slots[slot][0] == q_
    assert np.array_equal(got, want.astype(np.int64))
    assert orc.pair_nnz(plan) == int(want.sum())
    # canonical order and slot bookkeeping
    key = pairs[:, 0].astype(np.int64) * (len(kvb) + 1) + pairs[:, 1]
    assert np.all(np.diff(key) > 0)
    assert np.array_equal(pairs[:, 3], np.repeat(np.arange(len(slots)), slots[:, 2]))
    assert np.array_equal(slots[:, 1], np.concatenate([[0], np.cumsum(slots[:-1, 2])]))
    if c:
        assert slots[:, 2].max() <= c
    rows = np.concatenate([[0], np.cumsum(qb[slots[:, 0], 3])])
    assert np.array_equal(slots[:, 3], rows[:-1]) and plan["n_slot_rows"] == rows[-1]


def test_planner_rejects_bad_input():
    with pytest.raises(ValueError):
        orc.plan_blocks([4], 0)
    with pytest.raises(ValueError):
        orc.plan_blocks([-1], 4)
    with pytest.raises(ValueError):
        orc.plan_blocks([8], 4, 1, 0, [(0, 2)])
    with pytest.raises(ValueError):
        orc.plan_blocks([8], 4, 1, 0, [(0, 1), (0, 0)])


def test_flop_model():
    plan = orc.plan_blocks([8], 4, 1, 0)
    f, b = orc.flops(plan, 3, 16)
    assert f == 4 * 16 * 3 * 36 and b == 10 * 16 * 3 * 36


def test_bf16_decoding_matches_the_format():
    """bf16 = the upper 16 bits of an IEEE binary32: sign, 8 exponent bits (bias 127), 7 fraction
    bits.  Values the format itself fixes, then every one of the 65536 bit patterns against
    PyTorch's own bfloat16 decoding (independent code)."""
    fixed = {0x0000: 0.0, 0x3F80: 1.0, 0xBF80: -1.0, 0xC000: -2.0, 0x3FC0: 1.5, 0x4049: 3.140625, 0x3DCD: 0.10009765625,
             0x0001: 2.0 ** -133, 0x0080: 2.0 ** -126, 0x7F7F: (2.0 - 2.0 ** -7) * 2.0 ** 127,
             0x7F80: math.inf, 0xFF80: -math.inf}
    for bits, want in fixed.items():
        got = orc.bf16_to_f64(np.asarray([bits], dtype=np.uint16))
        assert got.dtype == np.float64 and got.shape == (1,)
        assert got[0] == want, (hex(bits), got[0], want)
    assert math.copysign(1.0, orc.bf16_to_f64(np.asarray([0x8000], dtype=np.uint16))[0]) == -1.0     # -0.0
    assert np.isnan(orc.bf16_to_f64(np.asarray([0x7FC0], dtype=np.uint16))[0])
    every = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    with np.errstate(invalid="ignore"):      # signalling NaN patterns are among them
        got = orc.bf16_to_f64(every.reshape(256, 256))
    want = torch.from_numpy(every.view(np.int16).copy()).view(torch.bfloat16).double().numpy().reshape(256, 256)
    assert got.shape == (256, 256)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan]) and np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))
    # the direct formula, element by element, on a sample of normal and subnormal patterns
    for bits in (0x0001, 0x007F, 0x0080, 0x1234, 0x3F81, 0x4A5B, 0x7F7F, 0x8001, 0xBEEF, 0xFF7F):
        sign, e, f = bits >> 15, (bits >> 7) & 0xFF, bits & 0x7F
        val = (f / 128.0) * 2.0 ** -126 if e == 0 else (1.0 + f / 128.0) * 2.0 ** (e - 127)
        assert orc.bf16_to_f64(np.asarray([bits], dtype=np.uint16))[0] == (-val if sign else val)


def test_input_generators_do_not_need_the_library():
    """The seeded generators serve the oracle and the library alike; importing them must not load
    the product's shared library (the oracle's pins run where it has not been built)."""
    import subprocess
    import sys
    code = ("import sys; from paper_2605_08524_amd import workloads; "
            "assert 'paper_2605_08524_amd.binding' not in sys.modules; "
            "import oracle.fcp_oracle; assert 'paper_2605_08524_amd.binding' not in sys.modules; print('ok')")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, "-c", code], cwd=root, capture_output=True, text=True)
    assert res.returncode == 0 and res.stdout.strip() == "ok", res.stderr


@pytest.mark.parametrize("bs,c,causal", [(4, 1, 1), (5, 2, 1), (3, 3, 0), (8, 0, 1)])
def test_stages_partition_the_plan_and_reduce_pairwise_to_the_whole(bs, c, causal):
    """A plan cut into execution stages: every pair lands in exactly one stage, stage k holds the k-th slot of each
    query block, and folding the stages' partial results one by one into a running (O, LSE), two at a time, gives
    the whole-sequence result (the reduction of the section "Context Parallelism" is associative)."""
    rng = np.random.default_rng(12)
    seq_lens = [13, 1, 8, 0, 21, 5]
    T, Hq, Hkv, d = sum(seq_lens), 4, 2, 8
    q, k, v = _bits(rng, T, Hq, d), _bits(rng, T, Hkv, d), _bits(rng, T, Hkv, d)
    plan = orc.plan_blocks(seq_lens, bs, causal, c)
    _, _, n_stages = orc.stage_tables(plan, 0)
    per_block = np.bincount(plan["slots"][:, 0], minlength=len(plan["q_blocks"]))
    assert n_stages == per_block.max()
    seen = []
    run_o = np.zeros((T, Hq, d))
    run_l = np.full((T, Hq), -np.inf)
    for st in range(n_stages + 1):
        sp, ss, _ = orc.stage_tables(plan, st)
        if st == n_stages:
            assert len(sp) == 0 and len(ss) == 0
            break
        assert len(ss) == int((per_block > st).sum())
        assert np.array_equal(ss[:, 3], plan["q_blocks"][ss[:, 0], 2])          # rows of the block itself
        assert np.array_equal(sp[:, 3], np.repeat(np.arange(len(ss)), ss[:, 2]))
        seen += [tuple(r[:3]) for r in sp]
        stage_plan = dict(plan, pairs=sp, slots=ss, n_slot_rows=T)
        op, lp = orc.partial_fwd(q, k, v, stage_plan, bs, causal)
        # two-way reduction through the same merge: "slot" 0 = the running result, slot 1 = this stage
        two = dict(plan, slots=np.asarray([(b, 0, 0, r0) for b in ss[:, 0] for r0 in (plan["q_blocks"][b][2], T + plan["q_blocks"][b][2])],
                                          dtype=np.int32).reshape(-1, 4))
        mo, ml = orc.merge_partials(np.concatenate([run_o, op]), np.concatenate([run_l, lp]), two)
        for b in ss[:, 0]:
            r0, n = int(plan["q_blocks"][b][2]), int(plan["q_blocks"][b][3])
            run_o[r0:r0 + n], run_l[r0:r0 + n] = mo[r0:r0 + n], ml[r0:r0 + n]
    assert sorted(seen) == sorted(tuple(r[:3]) for r in plan["pairs"])
    ow, lw = orc.worker_fwd(q, k, v, seq_lens, bs, causal)
    assert np.max(np.abs(run_o - ow)) < 1e-12
    assert np.max(np.abs(run_l - lw)) < 1e-12


def _visibility_from_tables(plan):
    """Dense count of how often every (Q-buffer row, KV-buffer row) entry is attended, read off the
    tables by the definitions of the pair kinds alone."""
    kvb, qb = plan["kv_blocks"], plan["q_blocks"]
    seg_id = {}
    for n, (kb, _, off, ln) in enumerate(plan["segments"]):
        ids = seg_id.setdefault(int(kb), np.full(int(kvb[kb][3]), -1))
        assert np.all(ids[off:off + ln] == -1)
        ids[off:off + ln] = n
    got = np.zeros((int(qb[:, 3].sum()), int(kvb[:, 3].sum())), dtype=np.int64)
    for q_, k_, kind, _ in plan["pairs"]:
        _, _, qs, ql = qb[q_]
        _, _, ks, kl = kvb[k_]
        blk = np.ones((ql, kl), dtype=np.int64)
        if kind in (orc.DIAG, orc.PACKED_DIAG):
            assert ql == kl
            blk = np.tril(blk)
        if kind in (orc.PACKED_FULL, orc.PACKED_DIAG):
            ids = seg_id[int(k_)]
            assert ql == kl and np.all(ids >= 0)          # members tile the block
            blk = blk * (ids[:, None] == ids[None, :])
        else:
            assert int(k_) not in seg_id                   # a packed block only pairs with itself
        got[qs:qs + ql, ks:ks + kl] += blk
    return got


@pytest.mark.parametrize("causal", [1, 0])
@pytest.mark.parametrize("owned_kind", ["all", "subset"])
def test_packed_planner_brute_force_coverage(causal, owned_kind):
    """The packed plan attends exactly the entries the definition names (same sequence, key not after the query
    under a causal mask), each once, once its rows are mapped back to the sequence-major order."""
    from oracle import fcp_sched_oracle as sch
    seq_lens, bs = [3, 10, 2, 0, 5, 17, 4, 1, 6, 8, 3], 8
    flat = orc.plan_blocks(seq_lens, bs, causal, 0)["kv_blocks"]
    unit, _, _ = sch.pack_units(flat, [int(b[3]) for b in flat], [0] * len(flat), bs)
    assert max(np.bincount(unit)) >= 3                     # the case has real packing
    q_owned = None
    if owned_kind == "subset":
        # drop the unit of block 0 as a whole, and one block of a long sequence
        drop = {b for b in range(len(flat)) if unit[b] == unit[0]} | {2}
        q_owned = np.asarray([(int(flat[b][0]), int(flat[b][1])) for b in range(len(flat)) if b not in drop], dtype=np.int32)
    plan = orc.plan_blocks_packed(seq_lens, bs, causal, 2, q_owned, unit)
    kv_src, q_src = orc.packed_row_maps(plan, seq_lens, bs, q_owned)
    T = sum(seq_lens)
    assert np.array_equal(np.sort(kv_src), np.arange(T))   # a permutation of the tokens
    assert len(set(q_src.tolist())) == len(q_src) == int(plan["q_blocks"][:, 3].sum())
    seq_of = np.repeat(np.arange(len(seq_lens)), seq_lens)
    pos_of = np.concatenate([np.arange(L) for L in seq_lens])
    # sequence-major Q rows: the owned tokens by (sequence, position)
    own_tok = np.arange(T) if q_owned is None else np.concatenate(
        [np.arange(bs * i, min(bs * (i + 1), seq_lens[s])) + int(np.sum(seq_lens[:s])) for s, i in q_owned])
    qs_, ks_ = own_tok[q_src], kv_src
    want = seq_of[qs_][:, None] == seq_of[ks_][None, :]
    if causal:
        want &= pos_of[ks_][None, :] <= pos_of[qs_][:, None]
    got = _visibility_from_tables(plan)
    assert np.array_equal(got, want.astype(np.int64))
    assert orc.pair_nnz(plan) == int(want.sum())
    # fewer blocks than without packing, one pair and one slot per packed query block
    assert len(plan["kv_blocks"]) < len(flat)
    packed_q = [q for q, _, kind, _ in plan["pairs"] if kind >= orc.PACKED_FULL]
    assert len(packed_q) == len(set(packed_q)) and len(packed_q) >= 1
    assert np.array_equal(plan["kv_blocks"][:, 2], np.concatenate([[0], np.cumsum(plan["kv_blocks"][:-1, 3])]))
    assert np.array_equal(plan["q_blocks"][:, 2], np.concatenate([[0], np.cumsum(plan["q_blocks"][:-1, 3])]))
    assert np.array_equal(plan["pairs"][:, 3], np.repeat(np.arange(len(plan["slots"])), plan["slots"][:, 2]))


def test_packed_planner_without_units_is_the_plain_planner():
    seq_lens, bs = [10, 3, 0, 17, 4, 1], 4
    for causal in (0, 1):
        for c in (0, 2):
            a = orc.plan_blocks(seq_lens, bs, causal, c)
            b = orc.plan_blocks_packed(seq_lens, bs, causal, c, None, None)
            for key in ("kv_blocks", "q_blocks", "pairs", "slots"):
                assert np.array_equal(a[key], b[key])
            assert a["n_slot_rows"] == b["n_slot_rows"] and len(b["segments"]) == 0
            b2 = orc.plan_blocks_packed(seq_lens, bs, causal, c, None, np.arange(len(a["kv_blocks"])))
            assert all(np.array_equal(a[k], b2[k]) for k in ("kv_blocks", "q_blocks", "pairs", "slots"))


def test_packed_planner_rejects_bad_units():
    with pytest.raises(ValueError):      # a block of a long sequence in a unit with another block
        orc.plan_blocks_packed([10, 2], 4, 1, 0, None, [0, 1, 2, 2])
    with pytest.raises(ValueError):      # the unit does not fit into a block
        orc.plan_blocks_packed([3, 3], 4, 1, 0, None, [0, 0])
    with pytest.raises(ValueError):      # a unit owned in part
        orc.plan_blocks_packed([2, 1, 5], 4, 1, 0, [(0, 0), (2, 0)], [0, 0, 1, 2])
    with pytest.raises(ValueError):      # one entry per unpacked block
        orc.plan_blocks_packed([2, 1], 4, 1, 0, None, [0])


def test_packed_attention_is_the_per_sequence_definition():
    """What a packed block computes is pinned to the plain definition without any planner: attention over the
    concatenated tokens of the members with a same-member (and causal) mask equals attention of every member by itself."""
    rng = np.random.default_rng(5)
    lens, H, d = [3, 1, 4], 2, 8
    q, k, v = (_rand(rng, sum(lens), H, d) for _ in range(3))
    member = np.repeat(np.arange(len(lens)), lens)
    for causal in (True, False):
        o_ref = np.zeros_like(q)
        lse_ref = np.zeros((sum(lens), H))
        off = 0
        for L in lens:
            o_ref[off:off + L], lse_ref[off:off + L] = orc.attention_fwd_seq(q[off:off + L], k[off:off + L], v[off:off + L], causal, 0.3)
            off += L
        for i in range(sum(lens)):       # row by row over the visible keys of the concatenation
            vis = [j for j in range(sum(lens)) if member[j] == member[i] and (not causal or j <= i)]
            o, lse = orc.attention_fwd_seq(q[i:i + 1], k[vis], v[vis], False, 0.3)
            assert np.allclose(o[0], o_ref[i], atol=1e-12) and np.allclose(lse[0], lse_ref[i], atol=1e-12)
