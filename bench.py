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

TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "cfg5_training_step_hbm_traffic.txt")


def measured_traffic(workload, kernel_instance):
    """HBM bytes per launch of `kernel_instance` (its full name, template arguments included) as recorded in the
    tracked rocprofv3 summary of the training step (FETCH_SIZE / WRITE_SIZE runs of this script, scaled by a plain copy
    of known size in the same runs).  None unless that file is about this workload and lists exactly this kernel
    instance: a figure carried over from a profile must not outlive the kernel it was measured on."""
    try:
        lines = open(TRAFFIC_PROFILE).read().splitlines()
    except OSError:
        return None
    if not any(l.startswith("workload: ") and l.split()[1] == workload for l in lines):
        return None
    for l in lines:
        if l.startswith(kernel_instance + " "):
            try:
                return float(l.split()[-1]) * 1e9       # last column: total GB
            except ValueError:
                return None
    return None


def pair_flops(plan, n_q_heads, head_dim):
    """Causal-adjusted FLOPs from the pair table: 4 d per unmasked score entry and query head
    forward (two contractions), 10 d backward (five)."""
    qlen = plan["q_blocks"][:, 3].astype("int64")
    klen = plan["kv_blocks"][:, 3].astype("int64")
    pr = plan["pairs"]
    m = qlen[pr[:, 0]]
    n = klen[pr[:, 1]]
    nnz = int(((pr[:, 2] == 0) * m * n + (pr[:, 2] == 1) * (m * (m + 1) // 2)).sum())
    if "segments" in plan and len(plan["segments"]):
        # packed blocks: their one pair attends every member sequence by itself
        causal = {int(kb): int(kind) & 1 for _, kb, kind, _ in pr if kind >= 2}
        for kb, _, _, ln in plan["segments"]:
            if int(kb) in causal:
                nnz += int(ln) * (int(ln) + 1) // 2 if causal[int(kb)] else int(ln) * int(ln)
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
    from paper_2605_08524_amd import FCP_FLAG_BWD_SPILL_DS, FCP_FLAG_DIRECT_SINGLE, FCP_FLAG_O_F32, workloads
    from paper_2605_08524_amd.harness import DevicePath

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream(dev)
    wl = workloads.make_workload(5, args.seed)
    spill = args.bwd == "spill"
    for bs in (256, 512, 1024, 2048, 4096, 8192):
        for c in (1, 4, 16, 0):
            wl.block_size, wl.coalesce = bs, c
            dp = DevicePath(wl, dev, flags=FCP_FLAG_DIRECT_SINGLE | FCP_FLAG_O_F32 | (FCP_FLAG_BWD_SPILL_DS if spill else 0),
                            backward=True, stream=stream)
            f_fwd, f_bwd, nnz = pair_flops(dp.plan, wl.n_q_heads, wl.head_dim)
            # four timed stages either way: forward, merge, then (D pass + dK/dV, dQ from dS) or (dQ with D, dK/dV)
            stages = [dp.fwd, dp.merge, (lambda: (dp.bwd_pre(), dp.bwd_dkdv())), dp.bwd_dq_ds] if spill else \
                     [dp.fwd, dp.merge, dp.bwd_dq_d, dp.bwd_dkdv]
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
                "backward": args.bwd,
                "nnz_per_head": nnz, "ms": {k: round(v, 3) for k, v in zip(("fwd", "merge", "bwd_pre+dkdv", "bwd_dq_ds") if spill else
                                                                           ("fwd", "merge", "bwd_dq", "bwd_dkdv"), ms)},
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


def merge_record(wl, dev, stream, steps, out_f32):
    """The merge where it is HBM-bound: the same batch at coalesce degree 1, so that every query block has one partial
    per KV block (3.5 GB of fp32 partials for the training batch, far beyond the 256 MB cache).  The forward fills the
    partials once; the merge alone is timed with events on the launch stream."""
    import numpy as np
    import torch
    from paper_2605_08524_amd import FCP_FLAG_O_F32
    from paper_2605_08524_amd.harness import DevicePath
    c_before = wl.coalesce
    wl.coalesce = 1
    try:
        dp = DevicePath(wl, dev, flags=FCP_FLAG_O_F32 if out_f32 else 0, backward=False, stream=stream)
    finally:
        wl.coalesce = c_before
    dp.fwd()
    dp.merge()
    torch.cuda.synchronize(dev)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for e0, e1 in evs:
        e0.record(stream)
        dp.merge()
        e1.record(stream)
    torch.cuda.synchronize(dev)
    ms = sum(e0.elapsed_time(e1) for e0, e1 in evs) / steps
    slots, qb = dp.plan["slots"], dp.plan["q_blocks"]
    cnt = np.bincount(slots[:, 0], minlength=len(qb))
    part_rows = int((cnt * qb[:, 3]).sum())
    rows = int(qb[:, 3].sum())
    nbytes = part_rows * wl.n_q_heads * (wl.head_dim * 4 + 4) + rows * wl.n_q_heads * (wl.head_dim * (4 if out_f32 else 2) + 4)
    rec = {"workload": f"{wl.name} at coalesce degree 1 ({len(slots)} partial slots)", "kernel": f"fcp::merge_kernel<{wl.head_dim}>",
           "algorithmic_bytes": nbytes, "ms": round(ms, 4), "achieved": round(nbytes / ms / 1e6, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
           "bound": "hbm", "frac": round(nbytes / ms / 1e6 / PEAK_HBM_GBS, 4),
           "traffic": measured_traffic(CONFIG5_NAME, f"fcp::merge_kernel<{wl.head_dim}>")}
    del dp
    torch.cuda.empty_cache()
    return rec


CONFIG5_NAME = "cfg5-training-step-fwd-bwd"


class PowerSampler:
    """Board power and shader clock from the driver's sysfs files (hwmon power1_input / power1_average in microwatts,
    pp_dpm_sclk's current level), sampled on a thread while a kernel runs in a loop."""

    def __init__(self):
        import glob
        self.power = self.sclk = self.cap = None
        for card in sorted(glob.glob("/sys/class/drm/card*/device")):
            hw = glob.glob(card + "/hwmon/hwmon*")
            for h in hw:
                for name in ("power1_input", "power1_average"):
                    if self.power is None and os.path.exists(os.path.join(h, name)):
                        self.power = os.path.join(h, name)
                if self.cap is None and os.path.exists(os.path.join(h, "power1_cap")):
                    self.cap = os.path.join(h, "power1_cap")
            if self.power and os.path.exists(os.path.join(card, "pp_dpm_sclk")):
                self.sclk = os.path.join(card, "pp_dpm_sclk")
                break
        self.rows, self.label, self.stop = [], None, False

    @staticmethod
    def _read(path):
        try:
            return open(path).read()
        except OSError:
            return ""

    def _loop(self):
        import re
        while not self.stop:
            if self.label is not None:
                try:
                    w = float(self._read(self.power)) / 1e6
                except ValueError:
                    w = float("nan")
                mhz = float("nan")
                for line in self._read(self.sclk).splitlines():
                    if line.rstrip().endswith("*"):
                        m = re.search(r"(\d+)\s*[Mm]hz", line)
                        if m:
                            mhz = float(m.group(1))
                self.rows.append((self.label, w, mhz))
            time.sleep(0.02)

    def start(self):
        import threading
        self.thread = threading.Thread(target=self._loop, daemon=True)
        self.thread.start()

    def mean(self, label):
        rows = [r for r in self.rows if r[0] == label]
        rows = rows[len(rows) // 3:]            # the clock needs a moment to settle on a new kind of load
        if not rows:
            return None, None
        return sum(r[1] for r in rows) / len(rows), sum(r[2] for r in rows) / len(rows)


def power_study(args):
    """Board power and shader clock while each kernel of the training step runs alone in a loop (about 2.5 s each), on
    the workload's N(0,1) operands and on all-zero operands, next to a pure MFMA stream and plain memory streams.
    Shows which kernels run into the board's power limit (the clock then pays for every joule the kernel spends).
    One JSON line per case."""
    import torch
    from paper_2605_08524_amd import (FCP_FLAG_BWD_SPILL_DS, FCP_FLAG_DIRECT_SINGLE, FCP_FLAG_O_F32, fcp_device_info, fcp_mfma_probe,
                                      workloads)
    from paper_2605_08524_amd.harness import DevicePath
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream(dev)
    ps = PowerSampler()
    if not ps.power or not ps.sclk:
        print(json.dumps({"error": "no hwmon power / pp_dpm_sclk files visible on this box"}))
        return
    wl = workloads.make_workload(5, args.seed)
    dp = DevicePath(wl, dev, flags=FCP_FLAG_DIRECT_SINGLE | FCP_FLAG_O_F32 | FCP_FLAG_BWD_SPILL_DS, backward=True, stream=stream)
    n_cu = fcp_device_info()["n_compute_units"]
    out = torch.zeros(8 * n_cu, dtype=torch.float32, device=dev)
    for fn in (dp.fwd, dp.merge, dp.bwd_pre, dp.bwd_dq_d, dp.bwd_dkdv, dp.bwd_dq_ds):
        fn()
    torch.cuda.synchronize(dev)
    f_fwd, f_bwd, nnz = pair_flops(dp.plan, wl.n_q_heads, wl.head_dim)
    unit = wl.head_dim * wl.n_q_heads * nnz
    src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    ps.start()
    time.sleep(1.5)
    cap_w = float(ps._read(ps.cap) or "nan") / 1e6 if ps.cap else None

    def run(label, fn, flops=None, nbytes=None, secs=2.5):
        time.sleep(0.8)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ps.label = label
        t0, n = time.time(), 0
        e0.record(stream)
        while time.time() - t0 < secs:
            for _ in range(10):
                fn()
            n += 10
            torch.cuda.synchronize(dev)
        e1.record(stream)
        torch.cuda.synchronize(dev)
        ps.label = None
        ms = e0.elapsed_time(e1) / n
        w, mhz = ps.mean(label)
        line = {"case": label, "ms_per_launch": round(ms, 4), "board_w": round(w, 1), "sclk_mhz": round(mhz), "power_cap_w": cap_w}
        if flops:
            line["executed_tflops"] = round(flops / ms / 1e9, 1)
            line["pj_per_executed_flop_above_idle"] = round((w - idle_w) * ms * 1e-3 / flops * 1e12, 3)
        if nbytes:
            line["gb_per_s"] = round(nbytes / ms / 1e6, 1)
            line["pj_per_byte_above_idle"] = round((w - idle_w) * ms * 1e-3 / nbytes * 1e12, 1)
        print(json.dumps(line), flush=True)

    ps.label = "idle"
    time.sleep(1.5)
    ps.label = None
    idle_w, idle_mhz = ps.mean("idle")
    print(json.dumps({"case": "idle", "board_w": round(idle_w, 1), "sclk_mhz": round(idle_mhz), "power_cap_w": cap_w}), flush=True)
    probe_flops = n_cu * 8 * 6000 * 16 * 32768.0
    run("mfma stream, zero operands", lambda: fcp_mfma_probe(0, 6000, out, stream), flops=probe_flops)
    run("mfma stream, random operands", lambda: fcp_mfma_probe(2, 6000, out, stream), flops=probe_flops)
    cases = [("fwd_kernel", dp.fwd, 4 * unit), ("dkdv_kernel, dS spilled", dp.bwd_dkdv, 8 * unit), ("dq_ds_kernel", dp.bwd_dq_ds, 2 * unit),
             ("dq_kernel (recomputing, with D)", dp.bwd_dq_d, 6 * unit)]
    for name, fn, fl in cases:
        run(name + ", N(0,1) operands", fn, flops=fl)
    run("delta_kernel", dp.bwd_pre, nbytes=wl.t_q * wl.n_q_heads * (wl.head_dim * 6 + 12))
    run("device copy 1 GiB (read + write)", lambda: dst.copy_(src), nbytes=2 * src.numel() * 4)
    run("device fill 1 GiB (write)", lambda: dst.fill_(1.5), nbytes=src.numel() * 4)
    for t in (dp.q, dp.k, dp.v, dp.d_o):
        t.fill_(0.0)
    torch.cuda.synchronize(dev)
    for name, fn, fl in cases:
        run(name + ", zero operands", fn, flops=fl)
    ps.stop = True


def probes(args):
    """Chip rates behind the kernels' design (include/fcp_probe.h): the matrix pipe with vector work beside it, LDS
    throughput per access pattern, fp32 atomic adds to memory.  One JSON line per case; rates per compute unit are
    given per nanosecond and, for reading against the LDS width, per cycle of the shader clock sampled during the case."""
    import torch
    from paper_2605_08524_amd import fcp_atomic_probe, fcp_device_info, fcp_lds_probe, fcp_mfma_valu_probe
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream(dev)
    n_cu = fcp_device_info()["n_compute_units"]
    ps = PowerSampler()
    sampling = bool(ps.power and ps.sclk)
    if sampling:
        ps.start()

    def timed(label, fn, min_s=1.0):
        fn()
        torch.cuda.synchronize(dev)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ps.label = label
        t0, n = time.time(), 0
        e0.record(stream)
        while time.time() - t0 < min_s:
            fn()
            n += 1
            torch.cuda.synchronize(dev)
        e1.record(stream)
        torch.cuda.synchronize(dev)
        ps.label = None
        w, mhz = ps.mean(label) if sampling else (None, None)
        return e0.elapsed_time(e1) / n, w, mhz

    out = torch.zeros(8 * n_cu, dtype=torch.float32, device=dev)
    for kind, kname in ((0, "zero"), (2, "random")):
        base = None
        for valu in (0, 2, 4, 6, 8, 12):
            iters = 20000
            ms, w, mhz = timed(f"mfma+{valu} {kname}", lambda: fcp_mfma_valu_probe(kind, valu, iters, out, stream))
            tf = n_cu * 8 * iters * 16 * 32768.0 / ms / 1e9
            base = base or tf
            print(json.dumps({"probe": "mfma stream with vector work", "operands": kname, "fp32_fma_per_mfma": valu, "ms": round(ms, 3),
                              "mfma_tflops": round(tf, 1), "relative_to_no_vector_work": round(tf / base, 3),
                              "board_w": w and round(w), "sclk_mhz": mhz and round(mhz)}), flush=True)
    idle_w = None
    if sampling:
        ps.label = "idle"
        time.sleep(1.0)
        ps.label = None
        idle_w, _ = ps.mean("idle")
    # random bytes: what an access costs in energy depends on how many bits toggle
    src = torch.randint(0, 256, (65536,), dtype=torch.uint8, device=dev)
    names = {0: ("ds_read_b128, swizzled rows", 1024), 1: ("ds_read_b64_tr_b16", 512), 2: ("ds_write_b128", 1024), 3: ("ds_write_b64", 512),
             4: ("LDS-DMA global_load_lds_dwordx4 (source in L2)", 1024)}
    for mode, (name, nbytes) in names.items():
        for waves in (4, 8):
            iters = 20000
            ms, w, mhz = timed(f"lds {mode} {waves}", lambda: fcp_lds_probe(mode, waves, iters, src, out, stream))
            per_cu = waves * iters * 16.0 * nbytes
            line = {"probe": "lds throughput per compute unit", "access": name, "waves": waves, "ms": round(ms, 3),
                    "bytes_per_ns": round(per_cu / ms / 1e6, 1), "sclk_mhz": mhz and round(mhz), "board_w": w and round(w)}
            if mhz:
                line["bytes_per_clk"] = round(per_cu / ms / 1e6 / (mhz / 1e3), 1)
            if w and idle_w:
                # whole-chip rate: every compute unit runs the same loop
                line["pj_per_byte_above_idle"] = round((w - idle_w) / (per_cu * n_cu / (ms * 1e-3)) * 1e12, 2)
            print(json.dumps(line), flush=True)
    n_rows, stride = 65536, 4096                 # 1 GiB of fp32: rows of 32 heads x 128
    buf = torch.zeros(n_rows * stride, dtype=torch.float32, device=dev)
    for wg in (1, 2, 4):
        iters = 2000
        ms, w, mhz = timed(f"atomic {wg}", lambda: fcp_atomic_probe(buf, n_rows, stride, iters, wg, stream), min_s=0.5)
        payload = n_cu * wg * 256 * iters * 16 * 4.0
        print(json.dumps({"probe": "fp32 atomic add to memory (dQ accumulation pattern)", "workgroups_per_cu": wg, "ms": round(ms, 3),
                          "payload_tb_per_s": round(payload / ms / 1e9, 3), "atomics_per_ns": round(payload / 4 / ms / 1e6, 1)}), flush=True)
    ps.stop = True


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
    ap.add_argument("--packed", action="store_true",
                    help="plan with fcp_plan_blocks_packed: the short sequences of a scheduling unit share one block")
    ap.add_argument("--with-backward", action="store_true", help="time the backward too on configs 2 to 4")
    ap.add_argument("--short-mix", action="store_true",
                    help="workload: 64K tokens of sequences shorter than a block (uniform [16, 256), block 1024) instead of --config; "
                         "with and without --packed it shows what sharing blocks is worth to the kernels")
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
    ap.add_argument("--running-merge", action="store_true",
                    help="forward-only configurations: run the forward as a loop over execution stages that fold their slots into a "
                         "running (O, LSE) in place (FCP_FLAG_RUNNING_MERGE; no partial buffers, no merge pass) and report its time "
                         "beside the one-pass path's")
    ap.add_argument("--heads", default=None, metavar="HQ/HKV",
                    help="override the head counts of the workload, e.g. 64/8 (the head shape of the paper's model)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (reads 1 GiB, writes 1 GiB): under rocprofv3 --pmc "
                         "its FETCH_SIZE / WRITE_SIZE give the scale factor for the kernels' HBM traffic")
    ap.add_argument("--sweep", action="store_true",
                    help="block size x coalesce degree sweep of the training step (one JSON line per point) instead of the benchmark line")
    ap.add_argument("--power", action="store_true",
                    help="board power and shader clock per kernel (sysfs sampling while each kernel loops), one JSON line per case, "
                         "instead of the benchmark line")
    ap.add_argument("--probes", action="store_true",
                    help="chip rates behind the kernels' design (MFMA with vector work beside it, LDS throughput per access "
                         "pattern, fp32 atomics), one JSON line per case, instead of the benchmark line")
    ap.add_argument("--no-merge-record", action="store_true",
                    help="skip the separate measurement of the merge kernel on the batch at coalesce degree 1")
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
    if args.power:
        power_study(args)
        return
    if args.probes:
        probes(args)
        return
    import torch
    from paper_2605_08524_amd import (FCP_FLAG_BWD_SPILL_DS, FCP_FLAG_DIRECT_SINGLE, FCP_FLAG_O_F32, FCP_FLAG_PART_BF16,
                                      fcp_device_info, workloads)
    from paper_2605_08524_amd.harness import DevicePath

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    wl = workloads.short_mix_workload(args.seed) if args.short_mix else workloads.make_workload(args.config, args.seed)
    if args.heads:
        wl.n_q_heads, wl.n_kv_heads = (int(x) for x in args.heads.split("/"))
        wl.name += f"-heads{wl.n_q_heads}x{wl.n_kv_heads}"
    backward = (args.config == 5 and not args.short_mix) or args.with_backward
    stream = torch.cuda.current_stream(dev)
    t0 = time.perf_counter()
    # a query block with one slot needs no reduction: the forward writes it straight to the final O / LSE
    flags = (0 if args.two_step else FCP_FLAG_DIRECT_SINGLE) | (FCP_FLAG_O_F32 if backward else 0)
    if args.bf16_partials:
        flags |= FCP_FLAG_PART_BF16
    spill = backward and args.bwd == "spill"
    if spill:
        flags |= FCP_FLAG_BWD_SPILL_DS
    dp = DevicePath(wl, dev, flags=flags, backward=backward, stream=stream, packed=args.packed)
    if args.packed:
        wl.name += "-packed"
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
    tf = "true" if spill else "false"
    kernel_instance = {"fwd": f"fcp::fwd_kernel<{wl.head_dim}, {'true' if args.packed else 'false'}>", "bwd_dkdv": f"fcp::dkdv_kernel<{wl.head_dim}, false, {tf}>",
                       "bwd_dq": f"fcp::dq_ds_kernel<{wl.head_dim}, false>" if spill else f"fcp::dq_kernel<{wl.head_dim}, true, false>"}
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
            "n_q_blocks": int(len(dp.plan["q_blocks"])), "packed_members": int(len(dp.plan.get("segments", ()))),
            "fwd_items": int(sum(-(-int(dp.plan["q_blocks"][qb][3]) // 128) for qb in dp.plan["slots"][:, 0]) * (wl.n_q_heads // 2 if (wl.n_q_heads // wl.n_kv_heads) % 2 == 0 else wl.n_q_heads)),
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
            "kernel_instance": kernel_instance[dom],
            "traffic": measured_traffic(wl.name, kernel_instance[dom]),
            "traffic_source": os.path.relpath(TRAFFIC_PROFILE, ROOT) + " (rocprofv3 FETCH_SIZE / WRITE_SIZE runs of this command; null if that file "
                              "does not list this kernel instance on this workload)",
            "avg_launch_ms": round(stage_ms[dom], 4),
        },
        "grid": info, "setup_s": round(setup_s, 2),
        "host_ms": {"plan_blocks": round(dp.plan_ms, 3), "queue_build": round(dp.queue_build_ms, 3)},
    }
    if args.config == 5 and not args.short_mix and not args.packed and not args.no_merge_record and not args.heads and args.inputs == "normal":
        # the merge launches nothing in the training configuration (one slot per query block): measured on its own
        out["merge"] = merge_record(wl, dev, stream, max(5, args.steps), out_f32=True)
    if args.running_merge and not backward:
        from paper_2605_08524_amd.harness import RunningPath
        part_bytes = dp.o_part.numel() * dp.o_part.element_size() + dp.lse_part.numel() * 4
        del dp
        torch.cuda.empty_cache()
        rp = RunningPath(wl, dev, stream=stream)
        rp.fwd()
        torch.cuda.synchronize(dev)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = max(2, min(args.steps, 5))
        e0.record(stream)
        for _ in range(reps):
            rp.fwd()
        e1.record(stream)
        torch.cuda.synchronize(dev)
        ms = e0.elapsed_time(e1) / reps
        out["running_merge"] = {"stages": rp.n_stages, "ms": round(ms, 3), "tflops": round(f_fwd / ms / 1e9, 1), "partial_bytes": 0,
                                "one_pass_partial_bytes": part_bytes, "one_pass_ms": round(stage_ms["fwd"] + stage_ms["merge"], 3)}
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
