#!/usr/bin/env python3
"""Benchmark of the LAQ re-eviction hot path (score -> select -> compact) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--no-cpu-baseline]

A step is one pass of the whole path (laq_evict) over every (sequence, layer) instance of the
workload, inputs resident in HBM.  Prints ONE JSON line: whole-job throughput in prefill
key-tokens scored+compacted per second per layer, the roofline of the dominant kernel
(algorithmic bytes / live HIP-event duration against 8 TB/s; its HBM traffic from two short
profiled child runs of the same command) and the CPU oracle timed on the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def algorithmic_bytes(cfg, budgets):
    """Bytes the method must move for one step, per stage (design notes: 'algorithmic bytes')."""
    e = cfg.elem_bytes
    n = cfg.n_inst
    k_stream = n * cfg.Hkv * cfg.L * cfg.d * e                    # K read once
    q_read = n * cfg.Hq * cfg.W * cfg.d * e
    scores_w = n * cfg.Hkv * cfg.L * 4
    score = k_stream + q_read + scores_w
    rows = sum(cfg.Hkv * min(b, cfg.L) for b in budgets)
    select = scores_w + rows * 4                                   # scores read, idx written
    compact = rows * 4 + 4 * rows * cfg.d * e                      # idx read; K',V' rows read + written
    return {"score": score, "select": select, "compact": compact, "total": score + select + compact}


def read_traffic(workload):
    """(HBM bytes per score-stage launch, where the figure comes from).  The bytes are not measured
    by this run: they are read from the committed rocprofv3 --pmc summary of the same command, if there
    is one for this workload; the source says so."""
    rel = os.path.join("profiles", "traffic_%s.txt" % workload)
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, "no committed counter summary for this workload"
    kernels = ""
    for line in open(path):
        if line.startswith("score_kernels="):
            kernels = line.split("=", 1)[1].strip()
        if line.startswith("traffic_bytes_per_launch="):
            return float(line.split("=", 1)[1]), ("%s (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this command, "
                                                  "recorded for the kernels: %s; not re-measured in this run)" % (rel, kernels))
    return None, "%s holds no traffic figure for the kernels of this build (see the note at its top)" % rel


SCORE_STAGE_KERNELS = ("stream_kernel", "row_constants", "reset_counters", "pool_boundaries", "fused_kernel",
                       "fused_reset", "stats_generic_kernel", "norm_generic_kernel", "pool_kernel")


DECODE_KERNELS = ("decode_kernel", "merge_parts_kernel")
LIVE_TRAFFIC_FAILED = []                   # why a profiled child run of this process failed, if one did


def live_traffic(args, cfg_id, kernels=SCORE_STAGE_KERNELS):
    """(HBM bytes per score-stage launch, source) measured now, or (None, why not).  Two short runs of this
    script as child processes under rocprofv3 (--pmc FETCH_SIZE, then WRITE_SIZE: one counter per run, 3
    steps each, same workload flags), each counter scaled by what it reads in the same run for a 1 GiB
    device-to-device copy; per kernel the average over its dispatches, summed over the kernels of the
    score stage.  The child runs start the single-read kernel with an ordinary launch
    (LAQ_COOPERATIVE_LAUNCH=0): a process profiled by rocprofv3 does not survive a cooperative one."""
    import csv
    import shutil
    import subprocess
    import tempfile
    if LIVE_TRAFFIC_FAILED:
        return None, "not measured in this run: %s" % LIVE_TRAFFIC_FAILED[0]
    if shutil.which("rocprofv3") is None:
        LIVE_TRAFFIC_FAILED.append("rocprofv3 not found")
        return None, "rocprofv3 not found"

    def failed(why):                       # one failure is enough: later workloads of the run do not try again
        LIVE_TRAFFIC_FAILED.append(why)
        return None, why
    flags = ["--config", str(cfg_id), "--window", args.window, "--pool-mode", args.pool_mode, "--layout", args.layout,
             "--path", args.path]
    env = dict(os.environ, TMPDIR="/tmp", LAQ_COOPERATIVE_LAUNCH="0")
    total, names = 0.0, []
    with tempfile.TemporaryDirectory(dir="/tmp") as tmp:
        for counter in ("FETCH_SIZE", "WRITE_SIZE"):
            out_dir = os.path.join(tmp, counter)
            cmd = ["rocprofv3", "--pmc", counter, "--output-format", "csv", "-d", out_dir, "-o", "t", "--",
                   sys.executable, os.path.abspath(__file__), "--no-cpu-baseline", "--no-probe", "--no-extra",
                   "--calibrate-copy", "--steps", "3", "--warmup", "1"] + flags
            try:
                res = subprocess.run(cmd, cwd="/tmp", env=env, capture_output=True, text=True, timeout=100)
            except (subprocess.TimeoutExpired, OSError) as err:
                return failed("profiled child run failed: %s" % type(err).__name__)
            if res.returncode != 0:
                return failed("profiled child run ended with status %d" % res.returncode)
            found = [os.path.join(d, f) for d, _, fs in os.walk(out_dir) for f in fs if f.endswith("counter_collection.csv")]
            if not found:
                return failed("the profiled child run left no counter file")
            per_kernel, copy = {}, 0.0
            for row in csv.DictReader(open(found[0])):
                if row["Counter_Name"] != counter:
                    continue
                name, val = row["Kernel_Name"], float(row["Counter_Value"])
                if "copyBuffer" in name:
                    copy = max(copy, val)
                elif "laq::" in name and any(k in name for k in kernels):
                    per_kernel.setdefault(name, []).append(val)
            if copy <= 0 or not per_kernel:
                return failed("the counter file holds no %s for the copy or for the kernels looked for" % counter)
            to_bytes = float(1 << 30) / copy            # the copy reads 1 GiB and writes 1 GiB
            total += sum(sum(v) / len(v) for v in per_kernel.values()) * to_bytes
            names = sorted(n.replace("void ", "").replace("(anonymous namespace)::", "").replace("laq::", "").split("(")[0]
                           for n in per_kernel)
    return float(round(total)), ("measured in this run: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE on two child runs of this command "
                   "(3 steps each), scaled by a 1 GiB device copy in the same runs; kernels: %s" % ", ".join(names))


SCORE_KERNEL_TEXT = {
    "single-read": "laq_score stage: fused_reset_kernel + fused_kernel (K read once; the unnormalised probabilities "
                   "stay in registers until the softmax denominators are known) + pool_boundaries_kernel",
    "two-pass": "laq_score stage: stream_kernel<pass 1> + row_constants_mfma_kernel + stream_kernel<pass 2> + "
                "pool_boundaries_kernel (K counted once in the algorithmic bytes, read twice)",
    "vector": "laq_score stage: vector-ALU kernels (K counted once in the algorithmic bytes, read twice)",
}


def bench_decode(args, torch, laq, cfg, budgets, dev):
    """One new token per instance attends to its compacted cache (packed K', V' of the config's budgets)."""
    n, dt = cfg.n_inst, cfg.torch_dtype
    total, _ = laq.packed_rows(budgets, cfg.Hkv, cfg.L)
    gen = torch.Generator(device=dev).manual_seed(1234)
    kc = torch.randn(total, cfg.d, generator=gen, device=dev).to(dt)
    vc = torch.randn(total, cfg.d, generator=gen, device=dev).to(dt)
    q = torch.randn(n, cfg.Hq, cfg.d, generator=gen, device=dev).to(dt)
    # the compacted caches of one step are smaller than the 256 MB last-level cache: the timed steps
    # walk through enough copies (> 1 GB in all) that every step reads its rows from HBM
    cache_bytes = 2 * total * cfg.d * cfg.elem_bytes
    copies = [(kc, vc)] + [(kc.clone(), vc.clone()) for _ in range(max(1, -(-(1 << 30) // cache_bytes)))]
    turn = [0]
    out_t = torch.empty(n, cfg.Hq, cfg.d, dtype=torch.float32, device=dev)
    ws = torch.empty(max(16, laq.laq_decode_workspace_bytes(n, cfg.Hq, cfg.Hkv, cfg.d, cfg.L, dt, budgets)),
                     dtype=torch.uint8, device=dev)

    def step():
        k_now, v_now = copies[turn[0] % len(copies)]
        turn[0] += 1
        laq.laq_decode_attention(q, k_now, v_now, budgets, cfg.Hkv, cfg.L, out=out_t, ws=ws)

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)                      # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    reps = max(3, min(args.steps, 20))
    ev[0].record()
    for _ in range(reps):
        step()
    ev[1].record()
    torch.cuda.synchronize()
    ms_kernel = ev[0].elapsed_time(ev[1]) / reps
    ab = 2 * total * cfg.d * cfg.elem_bytes + q.numel() * cfg.elem_bytes + out_t.numel() * 4
    achieved = ab / (ms_kernel * 1e-3) / 1e9
    workload = cfg.name + "+decode"
    traffic, traffic_source = None, None
    if not args.no_probe and not args.no_live_traffic:
        traffic, traffic_source = live_traffic(args, cfg.cfg_id, DECODE_KERNELS)
    if traffic is None:
        traffic, from_file = read_traffic(workload)
        traffic_source = from_file if traffic_source is None else "%s; %s" % (from_file, traffic_source)
    out = {
        "metric": "retained key-tokens attended/sec per layer (all heads)",
        "value": round(total / cfg.Hkv / (ms_per_step * 1e-3), 1), "unit": "key-tokens/s/layer", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": workload, "cfg_id": cfg.cfg_id, "instances": n, "Hq": cfg.Hq, "Hkv": cfg.Hkv,
                   "d": cfg.d, "L": cfg.L, "budget": cfg.budget, "packed_rows": total,
                   "cache_copies_cycled": len(copies)},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": "decode_kernel + merge_parts_kernel (K' and V' rows read once, q read, out written)",
                     "algorithmic_bytes_per_launch": ab, "ms_per_launch": round(ms_kernel, 4)},
    }
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        ids = list(range(n))                 # the oracle needs well under a second per instance here
        _, starts = laq.packed_rows(budgets, cfg.Hkv, cfg.L)
        t_cpu, rows = 0.0, 0
        for i in ids:
            bk = min(budgets[i], cfg.L)
            ki = kc[starts[i]:starts[i] + cfg.Hkv * bk].reshape(cfg.Hkv, bk, cfg.d).cpu()
            vi = vc[starts[i]:starts[i] + cfg.Hkv * bk].reshape(cfg.Hkv, bk, cfg.d).cpu()
            qi = q[i].cpu()
            c0 = time.perf_counter()
            oracle.decode_attention(qi, ki, vi)
            t_cpu += time.perf_counter() - c0
            rows += bk
        out["cpu_baseline"] = {"value": round(rows / t_cpu, 1), "unit": "key-tokens/s/layer", "cores": 1,
                               "kind": "oracle", "sample": "all %d instances, %.2f s" % (n, t_cpu)}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=4, help="workload: index into BASELINE.json configs (1-based)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-instances", type=int, default=0,
                    help="instances the CPU oracle is timed on, spread over the layers (about 2-5 s of one core "
                         "each); 0 (default): all of them")
    ap.add_argument("--cpu-threads", type=int, default=16, help="threads the CPU oracle's instances are spread over")
    ap.add_argument("--no-extra", action="store_true",
                    help="headline workload only: skip the batched 32k workload that the default run reports next to it")
    ap.add_argument("--path", choices=["evict", "decode"], default="evict",
                    help="evict (default): the re-eviction hot path, the headline workload; decode: one new "
                         "token's attention over the compacted cache of the same config (Sec. 4.3)")
    ap.add_argument("--window", choices=["trailing", "lookahead", "joined"], default="trailing",
                    help="observation window: the config's trailing window (default, the headline workload); "
                         "8 lookahead queries that see every key, nothing kept (Eq. 4); or 8 local window "
                         "queries joined with 8 lookahead queries, 8 keys kept (Eq. 5)")
    ap.add_argument("--pool-mode", choices=["max", "avg"], default="max",
                    help="sequence pooling: max (default, the headline workload) or the average of the "
                         "stage-1 eviction variant (Sec. 5.1)")
    ap.add_argument("--layout", choices=["dense", "token-major", "paged"], default="dense",
                    help="dense (default): k, v stored [n, Hkv, L, d]; token-major: stored [n, L, Hkv, d] and handed "
                         "over as strided views; paged: pools of 256-row blocks behind a shuffled block table")
    ap.add_argument("--no-probe", action="store_true",
                    help="skip the untimed extras -- the recall probe and the profiled child runs that measure "
                         "roofline.traffic -- (keeps profiler runs to the timed kernels)")
    ap.add_argument("--no-live-traffic", action="store_true",
                    help="take roofline.traffic from the committed counter summary instead of measuring it now")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device-to-device tensor copy (a kernel of known traffic, "
                         "for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU (every KV head is independent; nothing is sharded or "
              "exchanged) -- run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2505_20334_amd as laq
    from laq_inputs import CONFIGS, budgets_for, make_instance

    laq.load_library()                     # fails loudly if the HIP library is not built
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = CONFIGS[args.config]
    budgets = budgets_for(cfg)
    n = cfg.n_inst
    if args.path == "decode":
        return bench_decode(args, torch, laq, cfg, budgets, dev)
    out = measure_evict(args, torch, laq, cfg, budgets, dev, args.steps, args.warmup, primary=True)
    # the batched 32k workload next to the headline one (default run only): the same path on 8 sequences x 32
    # layers, 64 score rows per KV head
    if args.config == 4 and args.window == "trailing" and args.pool_mode == "max" and args.layout == "dense" \
            and not args.no_extra:
        torch.cuda.empty_cache()
        cfg5 = CONFIGS[5]
        extra = measure_evict(args, torch, laq, cfg5, budgets_for(cfg5), dev, min(args.steps, 10), min(args.warmup, 3),
                              primary=False)
        out["other_workloads"] = [{key: extra[key] for key in ("config", "value", "unit", "ms_per_step", "steps", "warmup",
                                                              "whole_path", "roofline")}]
    print(json.dumps(out))


def measure_evict(args, torch, laq, cfg, budgets, dev, steps, warmup, primary):
    """Times laq_evict on one workload; returns the JSON object of that workload."""
    from laq_inputs import make_instance
    n = cfg.n_inst
    q_pos, keep, workload = None, None, cfg.name
    if args.window != "trailing":
        import dataclasses
        if args.window == "lookahead":
            cfg = dataclasses.replace(cfg, W=8)
            q_pos, keep = [cfg.L + i for i in range(8)], 0
        else:
            cfg = dataclasses.replace(cfg, W=16)
            q_pos, keep = [cfg.L - 8 + i for i in range(8)] + [cfg.L + i for i in range(8)], 8
        workload = "%s+%s-window" % (cfg.name, args.window)
    if args.pool_mode != "max":
        workload += "+%s-pool" % args.pool_mode
    if args.layout != "dense":
        workload += "+%s" % args.layout

    # ---- inputs, generated on the device, resident before any timing ----
    dt = cfg.torch_dtype
    q = torch.empty(n, cfg.Hq, cfg.W, cfg.d, dtype=dt, device=dev)
    if args.layout != "token-major":
        k = torch.empty(n, cfg.Hkv, cfg.L, cfg.d, dtype=dt, device=dev)
        v = torch.empty(n, cfg.Hkv, cfg.L, cfg.d, dtype=dt, device=dev)
    else:
        k = torch.empty(n, cfg.L, cfg.Hkv, cfg.d, dtype=dt, device=dev).permute(0, 2, 1, 3)
        v = torch.empty(n, cfg.L, cfg.Hkv, cfg.d, dtype=dt, device=dev).permute(0, 2, 1, 3)
    for i in range(n):
        seq, layer = divmod(i, cfg.n_layer)
        qi, ki, vi, _ = make_instance(cfg, seq, layer, device=dev)
        q[i].copy_(qi); k[i].copy_(ki); v[i].copy_(vi)
    paged = {}
    k_in, v_in = k, v                       # what the library is handed (k, v stay dense for the CPU oracle)
    if args.layout == "paged":
        # the same rows in pools of 256-row blocks, the blocks of all instances shuffled
        br = 256
        per = -(-cfg.L // br)
        gen = torch.Generator(device="cpu").manual_seed(7)
        table = torch.randperm(n * per, generator=gen).reshape(n, per).int().to(dev)
        k_in = torch.zeros(n * per, cfg.Hkv, br, cfg.d, dtype=dt, device=dev)
        v_in = torch.zeros(n * per, cfg.Hkv, br, cfg.d, dtype=dt, device=dev)
        for i in range(n):
            for b in range(per):
                rows = min(br, cfg.L - b * br)
                k_in[table[i, b], :, :rows] = k[i, :, b * br:b * br + rows]
                v_in[table[i, b], :, :rows] = v[i, :, b * br:b * br + rows]
        paged = {"block_table": table, "L": cfg.L}
    total_rows, _ = laq.packed_rows(budgets, cfg.Hkv, cfg.L)
    scores = torch.empty(n, cfg.Hkv, cfg.L, dtype=torch.float32, device=dev)
    idx = torch.empty(total_rows, dtype=torch.int32, device=dev)
    k_out = torch.empty(total_rows, cfg.d, dtype=dt, device=dev)
    v_out = torch.empty(total_rows, cfg.d, dtype=dt, device=dev)
    ws = torch.empty(laq.laq_workspace_bytes(n, cfg.Hq, cfg.Hkv, cfg.d, cfg.L, cfg.W, dt, q_pos, keep),
                     dtype=torch.uint8, device=dev)
    keep_rows = cfg.W if keep is None else keep
    strides = (0, 0, 0) if k.is_contiguous() else (k.stride(0), k.stride(1), k.stride(2))
    score_kernel = laq.laq_score_kernel(n, cfg.Hq, cfg.Hkv, cfg.d, cfg.L, cfg.W, dt, q_pos, keep, strides,
                                        paged=(paged["block_table"], 256, k_in.stride(0)) if paged else None)

    def step():
        laq.laq_evict(q, k_in, v_in, budgets, cfg.pool, scores=scores, idx=idx, k_out=k_out, v_out=v_out, ws=ws,
                      q_pos=q_pos, keep=keep, pool_mode=args.pool_mode, **paged)

    if args.calibrate_copy and primary:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)                      # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    value = n * cfg.L / (ms_per_step * 1e-3)

    # ---- per-stage durations with events on the launch stream (torch's current stream) ----
    stages = {"score": 0.0, "select": 0.0, "compact": 0.0}
    reps = max(3, min(steps, 10))
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    for _ in range(reps):
        ev[0].record()
        laq.laq_score(q, k_in, cfg.pool, scores=scores, ws=ws, q_pos=q_pos, keep=keep, pool_mode=args.pool_mode, **paged)
        ev[1].record()
        laq.laq_select(scores, budgets, 1, keep_rows, idx=idx)
        ev[2].record()
        laq.laq_compact(k_in, v_in, idx, budgets, keep_rows, k_out=k_out, v_out=v_out, **paged)
        ev[3].record()
        torch.cuda.synchronize()
        stages["score"] += ev[0].elapsed_time(ev[1]) / reps
        stages["select"] += ev[1].elapsed_time(ev[2]) / reps
        stages["compact"] += ev[2].elapsed_time(ev[3]) / reps
    if laq.laq_workspace_status(ws, n, cfg.Hq, cfg.Hkv, cfg.d, cfg.L, cfg.W, dt) != 0:
        print("bench.py: the scoring kernel gave up a wait; the timings are not valid", file=sys.stderr)
        sys.exit(1)
    ab = algorithmic_bytes(cfg, budgets)
    achieved = ab["score"] / (stages["score"] * 1e-3) / 1e9
    traffic, traffic_source = None, None
    if not args.no_probe and not args.no_live_traffic:
        traffic, why = live_traffic(args, cfg.cfg_id)
        traffic_source = why
    if traffic is None:
        traffic, from_file = read_traffic(workload)
        traffic_source = from_file if traffic_source is None else "%s; %s" % (from_file, traffic_source)
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_source": traffic_source,
                "kernel": SCORE_KERNEL_TEXT[score_kernel],
                "algorithmic_bytes_per_launch": ab["score"],
                "ms_per_launch": round(stages["score"], 4)}

    out = {
        "metric": "prefill key-tokens scored+compacted/sec per layer (all heads)",
        "value": round(value, 1), "unit": "key-tokens/s/layer", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": workload, "cfg_id": cfg.cfg_id, "instances": n, "Hq": cfg.Hq, "Hkv": cfg.Hkv,
                   "d": cfg.d, "L": cfg.L, "W": cfg.W, "pool": cfg.pool, "budget": cfg.budget},
        "whole_path": {"algorithmic_GBs": round(ab["total"] / (ms_per_step * 1e-3) / 1e9, 1),
                       "frac_of_hbm_peak": round(ab["total"] / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                       "stage_ms": {s: round(t, 4) for s, t in stages.items()}},
        "roofline": roofline,
    }

    # quality probe in the spirit of Eq. 1-3 (untimed): how much of the selection made by all W window
    # queries (placed after the prompt, nothing kept) is recovered by the first quarter of them
    if primary and args.window == "trailing" and cfg.W >= 4 and not args.no_probe:
        see_all = [cfg.L] * cfg.W
        few = cfg.W // 4
        gold = laq.laq_evict(q, k, v, budgets, cfg.pool, q_pos=see_all, keep=0, pool_mode=args.pool_mode)[1]
        pred = laq.laq_evict(q[:, :, :few].contiguous(), k, v, budgets, cfg.pool, q_pos=see_all[:few], keep=0,
                             pool_mode=args.pool_mode)[1]
        _, rec = laq.laq_recall(pred, budgets, gold, budgets, cfg.Hkv, cfg.L)
        torch.cuda.synchronize()
        out["whole_path"]["recall_probe"] = {
            "value": round(float(rec.mean().item()), 4),
            "what": "mean over (instance, KV head) of |M_pred & M_gold| / |M_gold|: M_gold selected by all %d "
                    "window queries, M_pred by the first %d, every query after the prompt, synthetic data" % (cfg.W, few)}

    if primary and not args.no_cpu_baseline:
        # the oracle (plain C behind ctypes, which releases the interpreter lock) on every instance of the
        # workload, one instance per thread at a time
        from concurrent.futures import ThreadPoolExecutor
        import oracle
        oracle.build()
        m = n if args.cpu_instances <= 0 else max(1, min(args.cpu_instances, n))
        ids = sorted(set(round(i * (n - 1) / max(m - 1, 1)) for i in range(m)))      # spread over the layers
        threads = max(1, min(args.cpu_threads, len(ids), os.cpu_count() or 1))
        host = [(q[i].cpu(), k[i].cpu(), v[i].cpu()) for i in ids]

        def one(j):
            qi, ki, vi = host[j]
            oracle.evict(qi, ki, vi, budgets[ids[j]], cfg.pool, q_pos=q_pos, keep=keep, pool_mode=args.pool_mode)

        c0 = time.perf_counter()
        with ThreadPoolExecutor(threads) as pool:
            list(pool.map(one, range(len(ids))))
        t_cpu = time.perf_counter() - c0
        out["cpu_baseline"] = {"value": round(len(ids) * cfg.L / t_cpu, 1), "unit": "key-tokens/s/layer",
                               "cores": threads, "kind": "oracle",
                               "sample": "%s of the %d instances (all heads, full length), %d threads, %.1f s wall"
                                         % ("all" if len(ids) == n else "instances %s" % ids, n, threads, t_cpu)}
    return out


if __name__ == "__main__":
    main()
