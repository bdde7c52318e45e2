#!/usr/bin/env python3
"""Benchmark of the block-attention hot path on one MI355X.

A step = one pass of the whole path over one synthetic batch already resident in HBM:
forward partials (fcp_block_attn_fwd_out) -> merge (fcp_merge_partials) -> backward.  The backward is what
fcp_block_attn_bwd runs with FCP_FLAG_BWD_SPILL_DS (the default here): D = rowsum(dO o O) (fcp_bwd_preprocess) -> dK/dV,
which also leaves dS in the workspace (fcp_block_attn_bwd_dkdv) -> dQ = dS K (fcp_block_attn_bwd_dq_ds); with
--bwd recompute it is the variant without the flag: dQ kernel that recomputes S and dP and forms D itself
(fcp_block_attn_bwd_dq_d) -> dK/dV.  The default workload is the packed variable-length training step (64K tokens,
1024-token blocks, GQA 32/8, d = 128, bf16).

Prints ONE JSON line: whole-step throughput in causal-adjusted TFLOP/s, the roofline of the
dominant kernel measured with events on the launch stream, and the CPU oracle timed on a
bounded sample of the same workload (a reported baseline only).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6      # MI355X dense bf16 MFMA: 256 CUs x 4 SIMDs x 1024 FLOP/clk x 2.4 GHz
PEAK_HBM_GBS = 8000.0

# HBM bytes per launch, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script scaled by a
# plain copy of known size in the same runs (profiles/cfg5_training_step_hbm_traffic.txt); None
# for a workload or kernel that has not been measured.
MEASURED_TRAFFIC_BYTES = {
    ("cfg5-training-step-fwd-bwd", "fwd_kernel"): 2.781e9,
    ("cfg5-training-step-fwd-bwd", "dkdv_kernel"): 5.255e9,
    ("cfg5-training-step-fwd-bwd", "dq_kernel"): 4.430e9,
}


def pair_flops(plan, n_q_heads, head_dim):
    """Causal-adjusted FLOPs from the pair table: 4 d per unmasked score entry and query head
    forward (two contractions), 10 d backward (five)."""
    qlen = plan["q_blocks"][:, 3].astype("int64")
    klen = plan["kv_blocks"][:, 3].astype("int64")
    pr = plan["pairs"]
    m = qlen[pr[:, 0]]
    n = klen[pr[:, 1]]
    nnz = int(((pr[:, 2] == 0) * m * n + (pr[:, 2] == 1) * (m * (m + 1) // 2)).sum())
    return 4 * head_dim * n_q_heads * nnz, 10 * head_dim * n_q_heads * nnz, nnz


def cpu_baseline(wl, budget_s=20.0):
    """Time the fp64 oracle (forward + backward, whole sequences) on the shortest sequences of
    the workload until about `budget_s` seconds of CPU work are spent."""
    import numpy as np
    from oracle import fcp_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([int(i.get("num_threads", 1)) for i in threadpool_info()] + [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    q, k, v, do = wl.q(), wl.k(), wl.v(), wl.d_o()
    offs = np.concatenate([[0], np.cumsum(wl.seq_lens.astype(np.int64))])
    order = np.argsort(wl.seq_lens, kind="stable")
    spent, flops, used = 0.0, 0, []
    for s in order:
        L = int(wl.seq_lens[s])
        if L == 0:
            continue
        a, b = int(offs[s]), int(offs[s + 1])
        t0 = time.perf_counter()
        qs, ks, vs, ds = (orc.bf16_to_f64(x[a:b]) for x in (q, k, v, do))
        orc.attention_fwd_seq(qs, ks, vs, True)
        orc.attention_bwd_seq(qs, ks, vs, ds, True)
        spent += time.perf_counter() - t0
        flops += 14 * wl.head_dim * wl.n_q_heads * (L * (L + 1) // 2)
        used.append(L)
        if spent >= budget_s:
            break
    return {
        "value": round(flops / spent / 1e12, 6), "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
        "sample": f"fp64 numpy oracle fwd+bwd on the {len(used)} shortest sequences of the workload "
                  f"({sum(used)} tokens, {flops / 1e9:.1f} causal-adjusted GFLOP) in {spent:.1f} s",
    }


def sweep(args):
    """Throughput of the training step against block size and coalesce degree at fixed tokens: the
    paper's block-size study (its single-GPU attention efficiency collapses below 2K-token blocks
    and saturates above 4K; its system picks 4K blocks, coalesce degree 16) redone for this path,
    where one persistent launch covers all slots.  One JSON line per point."""
    import torch
    from paper_2605_08524_amd import FCP_FLAG_DIRECT_SINGLE, FCP_FLAG_O_F32, workloads
    from paper_2605_08524_amd.harness import DevicePath

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream(dev)
    wl = workloads.make_workload(5, args.seed)
    for bs in (256, 512, 1024, 2048, 4096, 8192):
        for c in (1, 4, 16, 0):
            wl.block_size, wl.coalesce = bs, c
            dp = DevicePath(wl, dev, flags=FCP_FLAG_DIRECT_SINGLE | FCP_FLAG_O_F32, backward=True, stream=stream)
            f_fwd, f_bwd, nnz = pair_flops(dp.plan, wl.n_q_heads, wl.head_dim)
            stages = [dp.fwd, dp.merge, dp.bwd_dq_d, dp.bwd_dkdv]
            for _ in range(args.warmup):
                for fn in stages:
                    fn()
            torch.cuda.synchronize(dev)
            evs = [[torch.cuda.Event(enable_timing=True) for _ in range(len(stages) + 1)] for _ in range(args.steps)]
            for s_ in range(args.steps):
                for i, fn in enumerate(stages):
                    evs[s_][i].record(stream)
                    fn()
                evs[s_][len(stages)].record(stream)
            torch.cuda.synchronize(dev)
            ms = [sum(evs[s_][i].elapsed_time(evs[s_][i + 1]) for s_ in range(args.steps)) / args.steps for i in range(len(stages))]
            step_ms = sum(ms)
            print(json.dumps({
                "block_size": bs, "coalesce": c, "n_pairs": int(len(dp.plan["pairs"])), "n_slots": int(len(dp.plan["slots"])),
                "nnz_per_head": nnz, "ms": {k: round(v, 3) for k, v in zip(("fwd", "merge", "bwd_dq", "bwd_dkdv"), ms)},
                "ms_per_step": round(step_ms, 3), "tflops": round((f_fwd + f_bwd) / step_ms / 1e9, 1),
                "fwd_tflops": round(f_fwd / (ms[0] + ms[1]) / 1e9, 1)}), flush=True)
            del dp
            torch.cuda.empty_cache()


def distribute(args):
    """Block distributor and congestion-free solver on the appendix's synthetic length traces: for each
    trace and worker count, the host time of the whole chain (block costs, greedy load-balanced
    assignment, data-flow edges, Delta sub-stages), the compute / memory / communication imbalance ratios
    ((max - mean) / max, as in the paper's balance study) and the oracle's time for the same steps where it
    finishes in seconds.  With a GPU, the most loaded worker's share of the 8-worker lognormal batch is
    then run forward + backward at its real shape.  One JSON line per point."""
    import numpy as np
    import paper_2605_08524_amd as fcp
    from oracle import fcp_sched_oracle as sch
    from paper_2605_08524_amd import workloads

    def ratio(x):
        x = np.asarray(x, dtype=np.float64)
        return round(float((x.max() - x.mean()) / x.max()), 4) if x.max() > 0 else 0.0

    bs, per_worker = 4096, 131072
    for kind in ("lognormal", "bimodal"):
        for n in (8, 32, 64, 128, 256):
            lens = workloads.length_trace(kind, n * per_worker, args.seed)
            t = [time.perf_counter()]
            blocks, mem, comp = fcp.fcp_block_costs(lens, bs, 1)
            t.append(time.perf_counter())
            owner, w_m, w_c = fcp.fcp_assign_blocks(mem, comp, n)
            t.append(time.perf_counter())
            edges = fcp.fcp_comm_edges(blocks, owner, n, 1)
            t.append(time.perf_counter())
            delta = fcp.fcp_solve_matchings(edges, n)
            t.append(time.perf_counter())
            stage, n_stages = fcp.fcp_coalesce_stages(edges, 16)
            t.append(time.perf_counter())
            line = {
                "trace": kind, "n_workers": n, "n_seqs": int(len(lens)), "n_blocks": int(len(blocks)), "block_size": bs,
                "imbalance": {"compute": ratio(w_c), "memory": ratio(w_m),
                              "send": ratio(np.bincount(edges[:, 0], minlength=n)), "recv": ratio(np.bincount(edges[:, 1], minlength=n))},
                "n_edges": int(len(edges)), "delta": int(delta), "stages_c16": int(n_stages),
                "host_ms": {k: round((b - a) * 1e3, 3) for k, a, b in zip(("costs", "assign", "edges", "solve", "coalesce"), t, t[1:])},
            }
            if n <= 64:       # the oracle's solver is the slow one: bounded to the sizes it finishes in seconds
                t0 = time.perf_counter()
                ob, om, oc = sch.block_costs(lens, bs, 1)
                o_owner, _, _ = sch.assign_blocks(om, oc, n)
                t1 = time.perf_counter()
                o_edges = sch.comm_edges(ob, o_owner, 1)
                o_stage, o_delta = sch.solve_matchings([e[0] for e in o_edges], [e[1] for e in o_edges], n)
                t2 = time.perf_counter()
                assert o_owner == owner.tolist() and o_delta == delta
                line["oracle_ms"] = {"costs+assign": round((t1 - t0) * 1e3, 1), "edges+solve": round((t2 - t1) * 1e3, 1)}
            print(json.dumps(line), flush=True)

    import torch
    if not torch.cuda.is_available():
        return
    from paper_2605_08524_amd.harness import DevicePath
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream(dev)
    n = 8
    lens = workloads.length_trace("lognormal", n * per_worker, args.seed)
    blocks, mem, comp = fcp.fcp_block_costs(lens, bs, 1)
    owner, w_m, w_c = fcp.fcp_assign_blocks(mem, comp, n)
    heavy = int(np.argmax(w_c))
    wl = workloads.custom_workload(lens, bs, causal=1, coalesce=16, n_q_heads=32, n_kv_heads=8, head_dim=128,
                                   q_owned=fcp.fcp_worker_blocks(blocks, owner, heavy), seed=args.seed, name="heaviest-share")
    dp = DevicePath(wl, dev, flags=fcp.FCP_FLAG_DIRECT_SINGLE | fcp.FCP_FLAG_O_F32, backward=True, stream=stream)
    f_fwd, f_bwd, nnz = pair_flops(dp.plan, wl.n_q_heads, wl.head_dim)
    assert nnz == int(w_c[heavy])
    stages = [dp.fwd, dp.merge, dp.bwd_dq_d, dp.bwd_dkdv]
    for _ in range(args.warmup):
        for fn in stages:
            fn()
    torch.cuda.synchronize(dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(args.steps):
        for fn in stages:
            fn()
    e1.record(stream)
    torch.cuda.synchronize(dev)
    ms = e0.elapsed_time(e1) / args.steps
    print(json.dumps({"share_of_worker": heavy, "n_workers": n, "trace": "lognormal", "tokens_q": int(w_m[heavy]),
                      "tokens_kv_resident": int(lens.sum()), "nnz_per_head": nnz, "n_pairs": int(len(dp.plan["pairs"])),
                      "ms_per_step": round(ms, 3), "tflops": round((f_fwd + f_bwd) / ms / 1e9, 1)}), flush=True)


def mfma_sustained(dev, stream):
    """What the matrix pipes sustain on a pure stream of the kernels' MFMA, by operand values
    (fcp_mfma_probe): the chip lowers its clock under the power drawn by random operands, so the
    rate it can hold on real data is well below the published peak that zeros reach."""
    import torch
    from paper_2605_08524_amd import fcp_device_info, fcp_mfma_probe
    n_cu = fcp_device_info()["n_compute_units"]
    out = torch.zeros(8 * n_cu, dtype=torch.float32, device=dev)
    res = {}
    for name, kind in (("zero_operands", 0), ("random_operands", 2)):
        iters = 60000                                   # 25-40 ms per launch
        fcp_mfma_probe(kind, iters // 4, out, stream)   # lets the clock settle for this kind of data
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        fcp_mfma_probe(kind, iters, out, stream)
        e1.record(stream)
        torch.cuda.synchronize(dev)
        res[name] = round(n_cu * 8 * iters * 16 * 32768.0 / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5, help="workload: 5 = training step (default), 2/3/4 = forward only")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--inputs", choices=("normal", "zeros", "half"), default="normal",
                    help="operand values: the workload's N(0,1) tensors (default: the benchmark), or all zeros / all 0.5 "
                         "(NOT a benchmark number: same instruction stream, shows how much the chip's clock depends on the data)")
    ap.add_argument("--no-mfma-probe", action="store_true",
                    help="skip the pure-MFMA measurement (sustained rate on zero / random operands) that is reported beside the roofline")
    ap.add_argument("--two-step", action="store_true",
                    help="every query block goes through the partial buffers and the merge, also those with one slot")
    ap.add_argument("--bf16-partials", action="store_true", help="keep the partial O buffer in bf16 (FCP_FLAG_PART_BF16)")
    ap.add_argument("--bwd", choices=("spill", "recompute"), default="spill",
                    help="backward variant: 'spill' keeps dS in the workspace (FCP_FLAG_BWD_SPILL_DS: D pass, dK/dV kernel that also "
                         "writes dS, streaming dQ kernel); 'recompute' runs the dQ kernel that recomputes S and dP, with D fused in")
    ap.add_argument("--heads", default=None, metavar="HQ/HKV",
                    help="override the head counts of the workload, e.g. 64/8 (the head shape of the paper's model)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (reads 1 GiB, writes 1 GiB): under rocprofv3 --pmc "
                         "its FETCH_SIZE / WRITE_SIZE give the scale factor for the kernels' HBM traffic")
    ap.add_argument("--sweep", action="store_true",
                    help="block size x coalesce degree sweep of the training step (one JSON line per point) instead of the benchmark line")
    ap.add_argument("--distribute", action="store_true",
                    help="block distributor + congestion-free solver study on synthetic length traces (host timings, "
                         "imbalance ratios; the most loaded worker's share on the GPU if there is one) instead of the benchmark line")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    if args.sweep:
        sweep(args)
        return
    if args.distribute:
        distribute(args)
        return
    import torch
    from paper_2605_08524_amd import (FCP_FLAG_BWD_SPILL_DS, FCP_FLAG_DIRECT_SINGLE, FCP_FLAG_O_F32, FCP_FLAG_PART_BF16,
                                      fcp_device_info, workloads)
    from paper_2605_08524_amd.harness import DevicePath

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    wl = workloads.make_workload(args.config, args.seed)
    if args.heads:
        wl.n_q_heads, wl.n_kv_heads = (int(x) for x in args.heads.split("/"))
        wl.name += f"-heads{wl.n_q_heads}x{wl.n_kv_heads}"
    backward = args.config == 5
    stream = torch.cuda.current_stream(dev)
    t0 = time.perf_counter()
    # a query block with one slot needs no reduction: the forward writes it straight to the final O / LSE
    flags = (0 if args.two_step else FCP_FLAG_DIRECT_SINGLE) | (FCP_FLAG_O_F32 if backward else 0)
    if args.bf16_partials:
        flags |= FCP_FLAG_PART_BF16
    spill = backward and args.bwd == "spill"
    if spill:
        flags |= FCP_FLAG_BWD_SPILL_DS
    dp = DevicePath(wl, dev, flags=flags, backward=backward, stream=stream)
    if args.inputs != "normal":
        for t in (dp.q, dp.k, dp.v) + ((dp.d_o,) if backward else ()):
            t.fill_(0.0 if args.inputs == "zeros" else 0.5)
    torch.cuda.synchronize(dev)
    setup_s = time.perf_counter() - t0
    f_fwd, f_bwd, nnz = pair_flops(dp.plan, wl.n_q_heads, wl.head_dim)
    step_flops = f_fwd + (f_bwd if backward else 0)

    stages = [("fwd", dp.fwd), ("merge", dp.merge)]
    if backward and spill:
        stages += [("bwd_pre", dp.bwd_pre), ("bwd_dkdv", dp.bwd_dkdv), ("bwd_dq", dp.bwd_dq_ds)]
    elif backward:
        stages += [("bwd_dq", dp.bwd_dq_d), ("bwd_dkdv", dp.bwd_dkdv)]

    def step(events=None):
        for i, (_, fn) in enumerate(stages):
            if events is not None:
                events[i][0].record(stream)
            fn()
            if events is not None:
                events[i][1].record(stream)

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize(dev)
        dst.copy_(src)
        torch.cuda.synchronize(dev)
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize(dev)
    evs = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in stages]
           for _ in range(args.steps)]
    torch.cuda.synchronize(dev)
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(evs[s])
    torch.cuda.synchronize(dev)
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    stage_ms = {}
    for i, (name, _) in enumerate(stages):
        stage_ms[name] = sum(evs[s][i][0].elapsed_time(evs[s][i][1]) for s in range(args.steps)) / args.steps

    # Each timed stage is exactly one kernel launch.  Algorithmic FLOPs per launch:
    # forward 2 contractions (4 d per unmasked entry and head), dK/dV kernel 4 (S, dP, dV, dK: 8 d),
    # dQ kernel 3 (S, dP, dQ: 6 d; S and dP are recomputed there instead of accumulating dQ with
    # atomics, so the backward executes 14 d per entry for an algorithmic 10 d).
    unit = wl.head_dim * wl.n_q_heads * nnz
    kernel_flops = {"fwd": 4 * unit, "bwd_dkdv": 8 * unit, "bwd_dq": (2 if spill else 6) * unit}
    kernel_name = {"fwd": "fwd_kernel", "bwd_dkdv": "dkdv_kernel", "bwd_dq": "dq_ds_kernel" if spill else "dq_kernel"}
    cands = [k for k in kernel_flops if k in stage_ms]
    dom = max(cands, key=lambda k: stage_ms[k])
    achieved = kernel_flops[dom] / (stage_ms[dom] * 1e-3) / 1e12
    p = dp.problem
    # the merge touches only query blocks with several slots (the others were written by the forward)
    import numpy as np
    slots, qb = dp.plan["slots"], dp.plan["q_blocks"]
    cnt = np.bincount(slots[:, 0], minlength=len(qb)) if len(slots) else np.zeros(len(qb), dtype=np.int64)
    merged = cnt > (1 if (flags & FCP_FLAG_DIRECT_SINGLE) else 0)
    merged_rows = int(qb[merged, 3].sum()) if len(qb) else 0
    part_rows = int((cnt[merged] * qb[merged, 3]).sum()) if len(qb) else 0
    merge_bytes = (part_rows * wl.n_q_heads * (wl.head_dim * (2 if (flags & FCP_FLAG_PART_BF16) else 4) + 4)
                   + merged_rows * wl.n_q_heads * (wl.head_dim * (4 if backward else 2) + 4))
    info = fcp_device_info()
    out = {
        "metric": "block-attention fwd+bwd TFLOP/s (causal-adj)" if backward else "block-attention fwd TFLOP/s (causal-adj)",
        "value": round(step_flops / (ms_per_step * 1e-3) / 1e12, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic" if args.inputs == "normal" else f"synthetic, all operands {args.inputs} (clock study, not a benchmark)",
        "config": {
            "workload": wl.name, "seed": args.seed, "tokens_q": p.t_q, "tokens_kv": p.t_kv,
            "block_size": wl.block_size, "coalesce": wl.coalesce, "n_q_heads": wl.n_q_heads,
            "n_kv_heads": wl.n_kv_heads, "head_dim": wl.head_dim, "n_seqs": int(len(wl.seq_lens)),
            "n_pairs": int(len(dp.plan["pairs"])), "n_slots": int(len(dp.plan["slots"])),
            "nnz_per_head": nnz, "o_dtype": "f32" if backward else "bf16", "parallelism": "single-gpu",
            "backward": (args.bwd if backward else None), "workspace_bytes": dp.ws_bytes,
        },
        "frac_of_bf16_peak": round(step_flops / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
        "stage_ms": {k: round(v, 4) for k, v in stage_ms.items()},
        "kernel_tflops": {k: round(kernel_flops[k] / stage_ms[k] / 1e9, 2) for k in cands},
        "merge_gbs": round(merge_bytes / stage_ms["merge"] / 1e6, 1) if merge_bytes else None,
        "merged_query_rows": merged_rows,
        "roofline": {
            "kernel": kernel_name[dom],
            "bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
            "traffic": MEASURED_TRAFFIC_BYTES.get((wl.name, kernel_name[dom])),
            "avg_launch_ms": round(stage_ms[dom], 4),
        },
        "grid": info, "setup_s": round(setup_s, 2),
        "host_ms": {"plan_blocks": round(dp.plan_ms, 3), "queue_build": round(dp.queue_build_ms, 3)},
    }
    if not args.no_mfma_probe:
        # context for the roofline, measured after the timed region: the published peak stays the denominator of "frac"
        sus = mfma_sustained(dev, stream)
        out["mfma_sustained_tflops"] = sus
        out["roofline"]["frac_of_sustained_random_operands"] = round(achieved / sus["random_operands"], 4)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl) if backward else None
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
