"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header
declares, plans blocks bit-exactly like the oracle, and reports errors as codes."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2605_08524_amd as fcp
from oracle import fcp_oracle as orc
from paper_2605_08524_amd import binding, workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = "".join(open(os.path.join(ROOT, "include", name)).read() for name in sorted(os.listdir(os.path.join(ROOT, "include"))))
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(fcp_[a-z_]+)\s*\(", hdr))
    assert declared == set(binding.EXPORTS)
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in declared:
        assert getattr(lib, name) is not None


def _same(plan_a, plan_b):
    for key in ("kv_blocks", "q_blocks", "pairs", "slots"):
        a, b = np.asarray(plan_a[key]).reshape(-1, 4), np.asarray(plan_b[key]).reshape(-1, 4)
        assert a.dtype == np.int32 and b.dtype == np.int32
        assert np.array_equal(a, b), key
    assert plan_a["n_slot_rows"] == plan_b["n_slot_rows"]


@pytest.mark.parametrize("config", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_plan_matches_oracle_on_configs(config, seed):
    wl = workloads.make_workload(config, seed)
    got = fcp.fcp_plan_blocks(wl.seq_lens, wl.block_size, wl.causal, wl.coalesce, wl.q_owned)
    want = orc.plan_blocks(wl.seq_lens, wl.block_size, wl.causal, wl.coalesce, wl.q_owned)
    _same(got, want)


def test_config3_pair_count():
    wl = workloads.make_workload(3, 0)
    plan = fcp.fcp_plan_blocks(wl.seq_lens, wl.block_size, wl.causal, wl.coalesce, wl.q_owned)
    # 32 zig-zag pairs (i, 511 - i): (i + 1) + (512 - i) = 513 KV blocks per pair of query blocks
    assert len(plan["pairs"]) == 32 * 513 and (plan["pairs"][:, 2] == 1).sum() == 64


@pytest.mark.parametrize("seq_lens,bs", [([1], 4), ([4], 4), ([5], 4), ([0, 0], 4), ([], 4), ([0, 7, 0, 1], 3),
                                         ([1000], 1), ([129, 128, 127], 128)])
@pytest.mark.parametrize("causal", [0, 1])
@pytest.mark.parametrize("c", [0, 1, 3, 16])
def test_plan_edge_cases(seq_lens, bs, causal, c):
    _same(fcp.fcp_plan_blocks(seq_lens, bs, causal, c), orc.plan_blocks(seq_lens, bs, causal, c))


def test_plan_owned_subsets_random():
    rng = np.random.default_rng(0)
    for _ in range(30):
        seq_lens = rng.integers(0, 60, size=rng.integers(1, 6))
        bs = int(rng.integers(1, 9))
        blocks = [(s, i) for s, L in enumerate(seq_lens) for i in range(-(-int(L) // bs))]
        keep = [b for b in blocks if rng.random() < 0.4]
        c = int(rng.integers(0, 4))
        causal = int(rng.integers(0, 2))
        owned = np.asarray(keep, dtype=np.int32).reshape(-1, 2)
        _same(fcp.fcp_plan_blocks(seq_lens, bs, causal, c, owned), orc.plan_blocks(seq_lens, bs, causal, c, owned))


def test_plan_error_codes():
    with pytest.raises(fcp.FcpError) as e:
        fcp.fcp_plan_blocks([4], 0)
    assert e.value.code == binding.FCP_ERR_INVALID_ARG
    with pytest.raises(fcp.FcpError) as e:
        fcp.fcp_plan_blocks([-3], 4)
    assert e.value.code == binding.FCP_ERR_INVALID_ARG
    with pytest.raises(fcp.FcpError) as e:
        fcp.fcp_plan_blocks([8], 4, 1, 0, [(0, 2)])
    assert e.value.code == binding.FCP_ERR_INVALID_ARG and "out of range" in str(e.value)
    with pytest.raises(fcp.FcpError) as e:
        fcp.fcp_plan_blocks([8], 4, 1, 0, [(0, 1), (0, 0)])
    assert e.value.code == binding.FCP_ERR_INVALID_ARG


def test_plan_capacity_too_small():
    lib = binding._lib
    sl = np.asarray([10, 3], dtype=np.int32)
    i32p = ctypes.POINTER(ctypes.c_int32)
    counts = [ctypes.c_int32(1) for _ in range(5)]
    tabs = [np.zeros((1, 4), dtype=np.int32) for _ in range(4)]
    rc = lib.fcp_plan_blocks(sl.ctypes.data_as(i32p), 2, 4, 1, 2, None, 0,
                             tabs[0].ctypes.data, ctypes.byref(counts[0]), tabs[1].ctypes.data, ctypes.byref(counts[1]),
                             tabs[2].ctypes.data, ctypes.byref(counts[2]), tabs[3].ctypes.data, ctypes.byref(counts[3]),
                             ctypes.byref(counts[4]))
    assert rc == binding.FCP_ERR_BUFFER_TOO_SMALL
    assert [c.value for c in counts] == [4, 4, 7, 5, 15]


def _problem(seq_lens=(300, 77), bs=128, hq=4, hkv=2, d=64, c=2):
    plan = fcp.fcp_plan_blocks(list(seq_lens), bs, 1, c)
    return fcp.Problem(plan, hq, hkv, d, bs)


def test_workspace_bytes_and_validation():
    assert fcp.fcp_workspace_bytes(_problem()) > 0
    with pytest.raises(fcp.FcpError) as e:
        fcp.fcp_workspace_bytes(_problem(d=96))
    assert e.value.code == binding.FCP_ERR_UNSUPPORTED
    with pytest.raises(fcp.FcpError) as e:
        fcp.fcp_workspace_bytes(_problem(hq=6, hkv=4))
    assert e.value.code == binding.FCP_ERR_UNSUPPORTED
    p = _problem()
    p.pairs[0, 2] = 7            # not a valid kind
    with pytest.raises(fcp.FcpError) as e:
        fcp.fcp_workspace_bytes(p)
    assert e.value.code == binding.FCP_ERR_INVALID_ARG
    p = _problem()
    p.pairs[1, 2] = 1            # FULL pair of different blocks relabelled DIAG
    with pytest.raises(fcp.FcpError) as e:
        fcp.fcp_workspace_bytes(p)
    assert e.value.code == binding.FCP_ERR_INVALID_ARG
    p = _problem()
    p.slots[1, 3] = 10 ** 6      # rows outside the partial buffers
    with pytest.raises(fcp.FcpError):
        fcp.fcp_workspace_bytes(p)


def test_null_pointers_are_rejected_before_any_launch():
    p = _problem()
    with pytest.raises(fcp.FcpError) as e:
        fcp.fcp_queue_build(p, 0, 1 << 20)
    assert e.value.code == binding.FCP_ERR_INVALID_ARG
    with pytest.raises(fcp.FcpError) as e:
        fcp.fcp_queue_build(p, 256, 8)
    assert e.value.code == binding.FCP_ERR_BUFFER_TOO_SMALL
    with pytest.raises(fcp.FcpError) as e:
        fcp.fcp_block_attn_fwd(p, 0, 0, 0, 0, 0, 0)
    assert e.value.code == binding.FCP_ERR_INVALID_ARG
    with pytest.raises(fcp.FcpError) as e:
        fcp.fcp_merge_partials(p, 0, 0, 0, 0, 0)
    assert e.value.code == binding.FCP_ERR_INVALID_ARG
    with pytest.raises(fcp.FcpError) as e:
        fcp.fcp_block_attn_bwd(p, *([0] * 10))
    assert e.value.code == binding.FCP_ERR_INVALID_ARG


def test_mfma_probe_rejects_bad_arguments_before_any_launch():
    for kind, iters, out in ((0, 10, 0), (0, 0, 256), (3, 10, 256), (-1, 10, 256)):
        with pytest.raises(fcp.FcpError) as e:
            fcp.fcp_mfma_probe(kind, iters, out)
        assert e.value.code == binding.FCP_ERR_INVALID_ARG


def test_workload_generators_are_seeded():
    a, b = workloads.make_workload(2, 0), workloads.make_workload(2, 0)
    assert np.array_equal(a.seq_lens, b.seq_lens) and a.seq_lens.sum() == 65536
    t1 = workloads.draw_tensor(0, 1, (100, 2, 8))
    t2 = workloads.draw_tensor(0, 1, (100, 2, 8))
    assert np.array_equal(t1, t2) and t1.dtype == np.uint16
    x = workloads.bf16_to_f32(t1)
    assert abs(float(x.mean())) < 0.1 and 0.9 < float(x.std()) < 1.1
    # round-to-nearest-even on a tie
    assert workloads.bf16_bits(np.asarray([1.00390625], dtype=np.float32))[0] == 0x3F80
    assert workloads.bf16_bits(np.asarray([1.01171875], dtype=np.float32))[0] == 0x3F82


@pytest.mark.parametrize("config", [1, 2, 3, 4])
def test_stage_tables_match_oracle(config):
    wl = workloads.make_workload(config, 1)
    if config == 1:
        wl.coalesce = 2
    plan = fcp.fcp_plan_blocks(wl.seq_lens, wl.block_size, wl.causal, wl.coalesce, wl.q_owned)
    ref_plan = orc.plan_blocks(wl.seq_lens, wl.block_size, wl.causal, wl.coalesce, wl.q_owned)
    _, n_stages = fcp.fcp_stage_tables(plan, 0)
    assert n_stages == orc.stage_tables(ref_plan, 0)[2]
    for st in sorted({0, 1, n_stages // 2, n_stages - 1, n_stages}):
        got, ns = fcp.fcp_stage_tables(plan, st)
        sp, ss, ref_ns = orc.stage_tables(ref_plan, st)
        assert ns == ref_ns
        assert np.array_equal(got["pairs"], sp) and np.array_equal(got["slots"], ss)
        assert got["n_slot_rows"] == int(ref_plan["q_blocks"][:, 3].sum())
        if len(ss):
            prob = fcp.Problem(got, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.block_size, 0.0,
                               binding.FCP_FLAG_RUNNING_MERGE | binding.FCP_FLAG_O_F32)
            assert fcp.fcp_workspace_bytes(prob) > 0            # a valid problem descriptor


def test_stage_tables_errors():
    plan = fcp.fcp_plan_blocks([300, 50], 128, 1, 1)
    with pytest.raises(fcp.FcpError) as e:
        fcp.fcp_stage_tables(plan, -1)
    assert e.value.code == binding.FCP_ERR_INVALID_ARG
    bad = dict(plan, slots=plan["slots"][::-1].copy())
    with pytest.raises(fcp.FcpError) as e:
        fcp.fcp_stage_tables(bad, 0)
    assert e.value.code == binding.FCP_ERR_INVALID_ARG


def _units(seq_lens, bs, causal):
    from oracle import fcp_sched_oracle as sch
    flat = orc.plan_blocks(seq_lens, bs, causal, 0)["kv_blocks"]
    return sch.pack_units(flat, [int(b[3]) for b in flat], [0] * len(flat), bs)[0] if len(flat) else None


def test_packed_plan_matches_oracle_random():
    """fcp_plan_blocks_packed against the oracle's packed planner, bit for bit, on random batches and shares."""
    rng = np.random.default_rng(11)
    for trial in range(150):
        bs = int(rng.choice([4, 8, 16]))
        sl = rng.integers(0, 3 * bs, size=int(rng.integers(1, 12)))
        causal, c = int(rng.integers(0, 2)), int(rng.choice([0, 1, 2, 3]))
        unit = _units(sl, bs, causal)
        qo = None
        if unit is not None and rng.random() < 0.5:
            flat = orc.plan_blocks(sl, bs, causal, 0)["kv_blocks"]
            keep = {u for u in set(unit) if rng.random() < 0.6}
            qo = np.asarray([(int(flat[b][0]), int(flat[b][1])) for b in range(len(flat)) if unit[b] in keep], dtype=np.int32).reshape(-1, 2)
        want = orc.plan_blocks_packed(sl, bs, causal, c, qo, unit)
        got = fcp.fcp_plan_blocks_packed(sl, bs, causal, c, qo, unit)
        for key in ("kv_blocks", "q_blocks", "pairs", "slots", "segments"):
            assert np.array_equal(want[key], got[key]), (trial, key)
        assert want["n_slot_rows"] == got["n_slot_rows"]


def test_packed_plan_on_the_multimodal_config():
    """Config 4 through block costs -> scheduling units -> packed plan, all in the library, against the same chain
    in the oracles; the packed plan has fewer query blocks and pairs than the plain one."""
    from paper_2605_08524_amd.harness import packed_plan
    wl = workloads.make_workload(4, 0)
    got = packed_plan(wl)
    want = orc.plan_blocks_packed(wl.seq_lens, wl.block_size, wl.causal, wl.coalesce, wl.q_owned,
                                  _units(wl.seq_lens, wl.block_size, wl.causal))
    for key in ("kv_blocks", "q_blocks", "pairs", "slots", "segments"):
        assert np.array_equal(want[key], got[key]), key
    plain = fcp.fcp_plan_blocks(wl.seq_lens, wl.block_size, wl.causal, wl.coalesce, wl.q_owned)
    assert len(got["q_blocks"]) < len(plain["q_blocks"]) and len(got["segments"]) > 0
    assert orc.pair_nnz(want) == orc.pair_nnz(orc.plan_blocks(wl.seq_lens, wl.block_size, wl.causal, wl.coalesce, wl.q_owned))
    prob = fcp.Problem(got, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.block_size)
    assert fcp.fcp_workspace_bytes(prob) > 0


def test_packed_plan_error_codes():
    def code(*a):
        with pytest.raises(fcp.FcpError) as e:
            fcp.fcp_plan_blocks_packed(*a)
        return e.value.code
    assert code([10, 2], 4, 1, 0, None, [0, 1, 2, 2]) == -1          # a block of a long sequence shares a unit
    assert code([3, 3], 4, 1, 0, None, [0, 0]) == -1                 # the unit does not fit into a block
    assert code([2, 1, 5], 4, 1, 0, [(0, 0), (2, 0)], [0, 0, 1, 2]) == -1   # a unit owned in part
    assert code([2, 1], 4, 1, 0, None, [0, 7]) == -1                 # unit index out of range
    assert code([2, 1], 4, 1, 0, None, None) == -1                   # blocks but no unit table


def test_segment_tables_are_validated():
    plan = fcp.fcp_plan_blocks_packed([3, 2, 9], 8, 1, 0, None, [0, 0, 1, 2])
    assert plan["segments"].tolist() == [[0, 0, 0, 3], [0, 1, 3, 2]] and plan["pairs"][0].tolist() == [0, 0, 3, 0]

    def rc(mutate):
        bad = {k: (v.copy() if hasattr(v, "copy") else v) for k, v in plan.items()}
        mutate(bad)
        with pytest.raises(fcp.FcpError) as e:
            fcp.fcp_workspace_bytes(fcp.Problem(bad, 2, 2, 64, 8))
        return e.value.code
    assert rc(lambda p: p["segments"].__setitem__((1, 3), 1)) == -1      # the members do not cover their block
    assert rc(lambda p: p["segments"].__setitem__((1, 2), 2)) == -1      # a gap between members
    assert rc(lambda p: p["pairs"].__setitem__((0, 2), 1)) == -1         # a DIAG pair on a block with members
    assert rc(lambda p: p["pairs"].__setitem__((1, 2), 3)) == -1         # a PACKED pair on a block without members
    assert rc(lambda p: p.__setitem__("segments", p["segments"][::-1].copy())) == -1   # not in (kv_blk, tok_off) order


def test_packed_block_size_limit():
    """The kernels keep a token's member bounds in two 16-bit halves: a packed block above 65 535 tokens is refused
    when the problem is validated (the planner itself has no such limit)."""
    plan = fcp.fcp_plan_blocks_packed([40000, 29000], 70000, 1, 0, None, [0, 0])
    assert plan["kv_blocks"].tolist() == [[0, 0, 0, 69000]] and len(plan["segments"]) == 2
    with pytest.raises(fcp.FcpError) as e:
        fcp.fcp_workspace_bytes(fcp.Problem(plan, 2, 2, 64, 70000))
    assert e.value.code == -3
    ok = fcp.fcp_plan_blocks_packed([40000, 25000], 70000, 1, 0, None, [0, 0])
    assert fcp.fcp_workspace_bytes(fcp.Problem(ok, 2, 2, 64, 70000)) > 0


@pytest.mark.parametrize("packed", [False, True])
def test_queue_tables_are_built_on_the_host_before_any_gpu_call(packed):
    """Without a GPU, fcp_queue_build still validates the problem, lays out the workspace and builds every table (work
    items, dependency lists, member bounds of packed blocks) in host memory; only the upload fails, with FCP_ERR_HIP.
    This is how the queue builder runs under the host sanitizers."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("needs a box without a GPU: here the upload would be attempted")
    from paper_2605_08524_amd.harness import packed_plan
    cases = [workloads.custom_workload([100, 156, 30, 70, 90, 700, 17], 256, 1, 2, 6, 2, 128, seed=1),
             workloads.custom_workload([33, 1, 200, 95, 700, 5, 129], 256, 0, 2, 4, 4, 64, seed=2),
             workloads.make_workload(4, 0)]
    for wl in cases:
        plan = packed_plan(wl) if packed else fcp.fcp_plan_blocks(wl.seq_lens, wl.block_size, wl.causal, wl.coalesce, wl.q_owned)
        for flags in (0, fcp.FCP_FLAG_DIRECT_SINGLE | fcp.FCP_FLAG_O_F32 | fcp.FCP_FLAG_BWD_SPILL_DS):
            prob = fcp.Problem(plan, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.block_size, 0.0, flags)
            nbytes = fcp.fcp_workspace_bytes(prob)
            with pytest.raises(fcp.FcpError) as e:
                fcp.fcp_queue_build(prob, 4096, nbytes)      # an aligned address that is never written: the upload cannot start
            assert e.value.code == -4, fcp.fcp_last_error()
